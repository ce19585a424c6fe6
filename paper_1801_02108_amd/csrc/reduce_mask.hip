// reduce_mask: binary computation mask -> ordered list of active blocks
// (Sec. 3.1 "Reduce mask to indices" and Sec. 3.4 "Fused downsample and indexing kernel" of
// arXiv 1801.02108).
//
// The paper appends indices with a global atomic counter, which gives an arbitrary order.
// Here the list is produced in lexicographic (n, by, bx) order without atomics, in two launches.
// Grids of at most 65 536 blocks (every configuration of the paper's detector is far below):
//   pass 1  rm_pool_blocks: one wavefront per block.  All loads of a window are issued at once (aligned
//           4-byte words where the mask allows), the lanes' partial pools are combined with cross-lane
//           moves, one lane thresholds and stores the block's flag byte.  No LDS, no barrier, no
//           branch around a load: the kernel is one memory round trip long;
//   pass 2  rm_compact_flags: one workgroup per 256 consecutive blocks counts the flags in front of
//           its run (16 flags per load) and compacts its own 256 by ballot + popcount.
// Larger grids (a count over all earlier flags per workgroup would grow quadratically):
//   pass 1  rm_pool_rows: one workgroup per block row, coalesced column pooling of the window rows
//           into LDS, then one thread per block pools its window columns, thresholds, stores a flag
//           byte and the row's number of active blocks;
//   pass 2  rm_compact: one workgroup per block row: exclusive prefix over the row counts, then
//           ballot + popcount compaction of the row's flags into the index list.
// The flag bytes of pass 1 are also what the fused consumers take (conv16.hip): they do the compaction
// of pass 2 in their own prologue, which saves a launch where a launch is a third of the step.
#include "common.h"

#include <mutex>

namespace sbnet {

constexpr int kRmThreads = 256;

__device__ __forceinline__ int wave_sum(int v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

// sum over the workgroup, result valid in every thread
__device__ __forceinline__ int block_sum(int v, int *lds /* >= 4 ints */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    return lds[0] + lds[1] + lds[2] + lds[3];
}

template <typename T> struct Vec4;
template <> struct Vec4<uint8_t> { typedef uchar4 type; };
template <> struct Vec4<float> { typedef float4 type; };

template <typename Acc> __device__ __forceinline__ Acc lowest_of();
template <> __device__ __forceinline__ int lowest_of<int>() { return (int)0x80000000; }
template <> __device__ __forceinline__ double lowest_of<double>() { return -__builtin_huge_val(); }

constexpr int kRmRows = 20;  // window rows loaded per batch: that many independent loads in flight
constexpr int kRmCols = 8;   // window columns read from LDS per batch

// VEC = 4: every thread pools four neighbouring columns with one 4-element load per row (needs
// W % 4 == 0); VEC = 1: any W.
template <typename T, typename Acc, int POOL, int VEC>
__global__ __launch_bounds__(kRmThreads) void rm_pool_rows(const T *__restrict__ mask, int H, int W,
                                                            sbnet_geom g, double threshold,
                                                            int32_t *__restrict__ rowcount,
                                                            uint8_t *__restrict__ flags) {
    extern __shared__ __align__(8) unsigned char lds_raw[];
    Acc *col = reinterpret_cast<Acc *>(lds_raw);
    __shared__ int red[4];
    typedef typename Vec4<T>::type V4;

    const int row = blockIdx.x;
    const int n = row / g.bcount_h, by = row - n * g.bcount_h;
    const int y0 = g.boffset_h + by * g.bstride_h;
    const int ylo = max(y0, 0), yhi = min(y0 + g.bsize_h, H);
    const bool rows_clipped = (y0 < 0) || (y0 + g.bsize_h > H);
    const Acc neutral = POOL == SBNET_POOL_AVG ? (Acc)0 : lowest_of<Acc>();

    // pool the window rows of every image column (consecutive threads -> consecutive columns)
    for (int x = threadIdx.x * VEC; x < W; x += kRmThreads * VEC) {
        Acc a[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) a[k] = neutral;
        const T *p0 = mask + ((size_t)n * H + ylo) * W + x;
        for (int yb = ylo; yb < yhi; yb += kRmRows, p0 += (size_t)kRmRows * W) {
            V4 q[kRmRows];
            T q1[kRmRows];
#pragma unroll
            for (int u = 0; u < kRmRows; ++u) {
                if (yb + u < yhi) {
                    if (VEC == 4) q[u] = *reinterpret_cast<const V4 *>(p0 + (size_t)u * W);
                    else q1[u] = p0[(size_t)u * W];
                }
            }
#pragma unroll
            for (int u = 0; u < kRmRows; ++u) {
                if (yb + u < yhi) {
                    Acc v[4];
                    if (VEC == 4) { v[0] = (Acc)q[u].x; v[1] = (Acc)q[u].y; v[2] = (Acc)q[u].z; v[3] = (Acc)q[u].w; }
                    else v[0] = (Acc)q1[u];
#pragma unroll
                    for (int k = 0; k < VEC; ++k) {
                        if (POOL == SBNET_POOL_AVG) a[k] += v[k];
                        else a[k] = v[k] > a[k] ? v[k] : a[k];
                    }
                }
            }
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if (POOL == SBNET_POOL_MAX && rows_clipped) a[k] = a[k] < (Acc)0 ? (Acc)0 : a[k];  // outside counts as 0
            col[x + k] = a[k];
        }
    }
    __syncthreads();

    int mine = 0;
    const double area = (double)g.bsize_h * (double)g.bsize_w;
    for (int bx = threadIdx.x; bx < g.bcount_w; bx += kRmThreads) {
        const int x0 = g.boffset_w + bx * g.bstride_w;
        const int xlo = max(x0, 0), xhi = min(x0 + g.bsize_w, W);
        const bool cols_clipped = (x0 < 0) || (x0 + g.bsize_w > W);
        Acc a = neutral;
        for (int xb = xlo; xb < xhi; xb += kRmCols) {
            Acc v[kRmCols];
#pragma unroll
            for (int u = 0; u < kRmCols; ++u) v[u] = col[min(xb + u, xhi - 1)];
#pragma unroll
            for (int u = 0; u < kRmCols; ++u) {
                if (xb + u < xhi) {
                    if (POOL == SBNET_POOL_AVG) a += v[u];
                    else a = v[u] > a ? v[u] : a;
                }
            }
        }
        if (POOL == SBNET_POOL_MAX && cols_clipped) a = a < (Acc)0 ? (Acc)0 : a;
        const double pooled = POOL == SBNET_POOL_AVG ? (double)a / area : (double)a;
        const int active = pooled > threshold ? 1 : 0;
        flags[(size_t)row * g.bcount_w + bx] = (uint8_t)active;
        mine += active;
    }
    const int total = block_sum(mine, red);
    if (threadIdx.x == 0) rowcount[row] = total;
}

__global__ __launch_bounds__(kRmThreads) void rm_compact(const int32_t *__restrict__ rowcount,
                                                          const uint8_t *__restrict__ flags, int rows,
                                                          int bcount_h, int bcount_w,
                                                          int32_t *__restrict__ indices,
                                                          int32_t *__restrict__ count, int cap) {
    __shared__ int red[4];
    __shared__ int wave_cnt[4];
    const int row = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // the first batch of flags travels together with the row counts
    const bool on0 = (int)threadIdx.x < bcount_w && flags[(size_t)row * bcount_w + threadIdx.x] != 0;
    int part = 0;
    for (int r = threadIdx.x; r < row; r += kRmThreads) part += rowcount[r];
    int base = block_sum(part, red);   // active blocks in all earlier rows

    const int n = row / bcount_h, by = row - n * bcount_h;
    for (int b0 = 0; b0 < bcount_w; b0 += kRmThreads) {
        const int bx = b0 + threadIdx.x;
        const bool on = b0 == 0 ? on0 : (bx < bcount_w && flags[(size_t)row * bcount_w + bx] != 0);
        const unsigned long long ballot = __ballot(on);
        __syncthreads();
        if (lane == 0) wave_cnt[wave] = __popcll(ballot);
        __syncthreads();
        int before = 0;
        for (int w = 0; w < wave; ++w) before += wave_cnt[w];
        if (on) {
            const int pos = base + before + __popcll(ballot & ((1ull << lane) - 1ull));
            if (pos < cap) {
                indices[3 * (size_t)pos + 0] = n;
                indices[3 * (size_t)pos + 1] = by;
                indices[3 * (size_t)pos + 2] = bx;
            }
        }
        base += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    }
    if (row == rows - 1 && threadIdx.x == 0) *count = base;
}

// ---- grids of at most kFlagPathMaxBlocks blocks ---------------------------------------------------------------

// Sum (or max) of a non-negative int over the 64 lanes, result in lane 63: four shifts inside the rows of 16
// lanes, then the row totals are passed on to the next row and to the upper half (cross-lane moves in the
// VALU's data path: no LDS round trips).  Lanes without a source read 0, the identity of both operations here.
template <int POOL>
__device__ __forceinline__ int wave_pool_nonneg(int v) {
#define SBNET_RM_STEP(CTRL, ROWS)                                                                     \
    {                                                                                                 \
        const int o = __builtin_amdgcn_update_dpp(0, v, CTRL, ROWS, 0xf, false);                      \
        v = POOL == SBNET_POOL_AVG ? v + o : (o > v ? o : v);                                          \
    }
    SBNET_RM_STEP(0x111, 0xf)   // row_shr:1
    SBNET_RM_STEP(0x112, 0xf)   // row_shr:2
    SBNET_RM_STEP(0x114, 0xf)   // row_shr:4
    SBNET_RM_STEP(0x118, 0xf)   // row_shr:8      lane 15 of every row: the row's pool
    SBNET_RM_STEP(0x142, 0xa)   // row_bcast:15   rows 1 and 3 take in the row before them
    SBNET_RM_STEP(0x143, 0xc)   // row_bcast:31   rows 2 and 3 take in lane 31: lane 63 holds everything
#undef SBNET_RM_STEP
    return v;
}

template <typename Acc, int POOL>
__device__ __forceinline__ Acc wave_pool_any(Acc v) {
    for (int o = 32; o > 0; o >>= 1) {
        const Acc u = __shfl_xor(v, o, 64);
        v = POOL == SBNET_POOL_AVG ? v + u : (u > v ? u : v);
    }
    return v;
}

constexpr int kFlagPathMaxBlocks = 65536;
constexpr int kPoolUnroll = 4;       // loads a lane keeps in flight per batch

struct BlockDivs {
    FastDiv per_sample, per_row;     // blocks per sample, blocks per block row
};

// WORDS: T is uint8_t, W % 4 == 0 and the mask is 4-byte aligned: a lane loads aligned words that cover the
// window's columns and leaves out the bytes beside it.  Otherwise one element per load.
template <typename T, typename Acc, int POOL, bool WORDS>
__global__ __launch_bounds__(kRmThreads) void rm_pool_blocks(const T *__restrict__ mask, int H, int W, sbnet_geom g,
                                                              BlockDivs dv, int total, double threshold,
                                                              uint8_t *__restrict__ flags) {
    const int lane = threadIdx.x & 63;
    const int blk = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (kRmThreads / 64) + (threadIdx.x >> 6)));
    if (blk >= total) {                                       // uniform over the wavefront
        if (blk < ((total + 15) & ~15) && lane == 0) flags[blk] = 0;     // the padding up to a multiple of 16 reads as inactive
        return;
    }
    const int n = (int)fdiv((uint32_t)blk, dv.per_sample);
    const int rem = blk - n * g.bcount_h * g.bcount_w;
    const int by = (int)fdiv((uint32_t)rem, dv.per_row), bx = rem - by * g.bcount_w;
    const int y0 = g.boffset_h + by * g.bstride_h, x0 = g.boffset_w + bx * g.bstride_w;
    const int ylo = max(y0, 0), yhi = min(y0 + g.bsize_h, H);
    const int xlo = max(x0, 0), xhi = min(x0 + g.bsize_w, W);
    const bool clipped = y0 < 0 || x0 < 0 || y0 + g.bsize_h > H || x0 + g.bsize_w > W;
    const Acc neutral = POOL == SBNET_POOL_AVG ? (Acc)0 : lowest_of<Acc>();
    Acc a = neutral;
    if (yhi > ylo && xhi > xlo) {                             // uniform: the window meets the image
        const int per_row = WORDS ? ((xhi + 3) >> 2) - (xlo >> 2) : xhi - xlo;     // loads per window row
        const int first = WORDS ? (xlo >> 2) : xlo;
        const int count = per_row * (yhi - ylo);
        const size_t row_units = WORDS ? (size_t)(W >> 2) : (size_t)W;
        const size_t base = ((size_t)n * H + ylo) * row_units + first;
        for (int i0 = 0; i0 < count; i0 += 64 * kPoolUnroll) {
            uint32_t wv[kPoolUnroll];
            T ev[kPoolUnroll];
            int col[kPoolUnroll];
#pragma unroll
            for (int u = 0; u < kPoolUnroll; ++u) {            // every load is issued (index clamped), none waits
                const int i = min(i0 + u * 64 + lane, count - 1);
                const int r = i / per_row, c = i - r * per_row;
                col[u] = first + c;
                if (WORDS) wv[u] = reinterpret_cast<const uint32_t *>(mask)[base + (size_t)r * row_units + c];
                else ev[u] = mask[base + (size_t)r * row_units + c];
            }
#pragma unroll
            for (int u = 0; u < kPoolUnroll; ++u) {
                const bool live = i0 + u * 64 + lane < count;
                if (WORDS) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int x = col[u] * 4 + k;
                        const Acc v = (live && x >= xlo && x < xhi) ? (Acc)((wv[u] >> (8 * k)) & 0xffu) : neutral;
                        a = POOL == SBNET_POOL_AVG ? a + v : (v > a ? v : a);
                    }
                } else {
                    const Acc v = live ? (Acc)ev[u] : neutral;
                    a = POOL == SBNET_POOL_AVG ? a + v : (v > a ? v : a);
                }
            }
        }
    }
    if (sizeof(Acc) == 4) {       // integer pools of a u8 mask: never negative, identity 0
        a = (Acc)wave_pool_nonneg<POOL>((int)(POOL == SBNET_POOL_AVG ? a : (a < (Acc)0 ? (Acc)0 : a)));
    } else {
        a = wave_pool_any<Acc, POOL>(a);
    }
    if (lane == 63) {
        if (POOL == SBNET_POOL_MAX && clipped) a = a < (Acc)0 ? (Acc)0 : a;      // outside counts as 0
        const double area = (double)g.bsize_h * (double)g.bsize_w;
        const double pooled = POOL == SBNET_POOL_AVG ? (double)a / area : (double)a;
        flags[blk] = pooled > threshold ? (uint8_t)1 : (uint8_t)0;
    }
}

// The common case, tuned for latency: u8 mask, W % 4 == 0, 4-byte aligned.  A lane owns one aligned word of
// one window row per batch: LP = 2^lp_shift lanes side by side cover a row's words, 64 / LP rows per batch.
// Bytes beside the window are cleared with one AND; the sum of a word's bytes is one instruction.  The
// threshold is an integer cutoff worked out on the host (smallest pool value that counts as active), so
// the decision needs no division here and is the same decision bit for bit.
template <int POOL>
__global__ __launch_bounds__(kRmThreads) void rm_pool_blocks_u8w(const uint32_t *__restrict__ mask, int H, int W4,
                                                                  sbnet_geom g, BlockDivs dv, int total, int lp_shift,
                                                                  int cutoff, uint8_t *__restrict__ flags) {
    const int lane = threadIdx.x & 63;
    const int blk = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (kRmThreads / 64) + (threadIdx.x >> 6)));
    if (blk >= total) {                                       // uniform over the wavefront
        if (blk < ((total + 15) & ~15) && lane == 0) flags[blk] = 0;     // the padding up to a multiple of 16 reads as inactive
        return;
    }
    const int n = (int)fdiv((uint32_t)blk, dv.per_sample);
    const int rem = blk - n * g.bcount_h * g.bcount_w;
    const int by = (int)fdiv((uint32_t)rem, dv.per_row), bx = rem - by * g.bcount_w;
    const int y0 = g.boffset_h + by * g.bstride_h, x0 = g.boffset_w + bx * g.bstride_w;
    const int ylo = max(y0, 0), yhi = min(y0 + g.bsize_h, H);
    const int xlo = max(x0, 0), xhi = min(x0 + g.bsize_w, W4 * 4);
    int a = 0;
    if (yhi > ylo && xhi > xlo) {                             // uniform: the window meets the image
        const int w_lo = xlo >> 2, w_hi = (xhi - 1) >> 2;     // first and last word of a window row
        const int lp = 1 << lp_shift;
        const int c = lane & (lp - 1), r = lane >> lp_shift, rows_per = 64 >> lp_shift;
        const uint32_t *base = mask + ((size_t)n * H) * W4;
        for (int c0 = w_lo; c0 <= w_hi; c0 += lp) {
            const int wc = c0 + c;
            // bytes of word wc inside [xlo, xhi)
            uint32_t keep = 0xffffffffu;
            if (wc == w_lo) keep &= 0xffffffffu << (8 * (xlo & 3));
            if (wc == w_hi) keep &= 0xffffffffu >> (8 * (3 - ((xhi - 1) & 3)));
            if (wc > w_hi) keep = 0u;
            const int wcl = min(wc, w_hi);
            for (int r0 = ylo; r0 < yhi; r0 += rows_per * kPoolUnroll) {
                uint32_t q[kPoolUnroll];
#pragma unroll
                for (int u = 0; u < kPoolUnroll; ++u)            // clamped: every load is issued, none waits
                    q[u] = base[(size_t)min(r0 + u * rows_per + r, yhi - 1) * W4 + wcl];
#pragma unroll
                for (int u = 0; u < kPoolUnroll; ++u) {
                    const uint32_t w = (r0 + u * rows_per + r < yhi) ? (q[u] & keep) : 0u;
                    if (POOL == SBNET_POOL_AVG) {
                        a = (int)__builtin_amdgcn_sad_u8(w, 0u, (uint32_t)a);
                    } else {
                        const uint32_t m01 = max(w & 0xffu, (w >> 8) & 0xffu), m23 = max((w >> 16) & 0xffu, w >> 24);
                        a = max(a, (int)max(m01, m23));
                    }
                }
            }
        }
    }
    a = wave_pool_nonneg<POOL>(a);
    if (lane == 63) flags[blk] = a >= cutoff ? (uint8_t)1 : (uint8_t)0;
}

// flags: one byte per block in lexicographic order, padded to a multiple of 16 bytes (the padding is never counted)
__global__ __launch_bounds__(kRmThreads) void rm_compact_flags(const uint8_t *__restrict__ flags, int total, sbnet_geom g,
                                                                BlockDivs dv, int32_t *__restrict__ indices,
                                                                int32_t *__restrict__ count, int cap) {
    __shared__ int red[4];
    __shared__ int wave_cnt[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int start = blockIdx.x * kRmThreads;                // first block of this workgroup's run (multiple of 16)
    const int blk = start + (int)threadIdx.x;
    const bool on = blk < total && flags[blk] != 0;           // travels together with the loads of the count
    int part = 0;
    for (int v = threadIdx.x; v * 16 < start; v += kRmThreads)
        part += __popc(nonzero_bytes16(reinterpret_cast<const uint4 *>(flags)[v], 16));
    const int base = block_sum(part, red);                    // active blocks in front of the run
    const unsigned long long ballot = __ballot(on);
    if (lane == 0) wave_cnt[wave] = __popcll(ballot);
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += wave_cnt[w];
    if (on) {
        const int pos = base + before + __popcll(ballot & ((1ull << lane) - 1ull));
        if (pos < cap) {
            const int n = (int)fdiv((uint32_t)blk, dv.per_sample);
            const int rem = blk - n * g.bcount_h * g.bcount_w;
            const int by = (int)fdiv((uint32_t)rem, dv.per_row);
            indices[3 * (size_t)pos + 0] = n;
            indices[3 * (size_t)pos + 1] = by;
            indices[3 * (size_t)pos + 2] = rem - by * g.bcount_w;
        }
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) *count = base + wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
}

}  // namespace sbnet

using namespace sbnet;

static size_t rowcount_bytes(int rows) { return (((size_t)rows * 4) + 15) & ~(size_t)15; }

extern "C" size_t sbnet_workspace_bytes(int N, const sbnet_geom *g) {
    if (N <= 0 || !geom_ok(g)) return 0;
    const size_t rows = (size_t)N * g->bcount_h;
    return rowcount_bytes((int)rows) + ((rows * g->bcount_w + 15) & ~(size_t)15);
}

namespace sbnet {

static sbnet_status check_mask_args(const char *who, const void *mask, sbnet_dtype mdt, int N, int H, int W,
                                    const sbnet_geom *g, sbnet_pool pool) {
    if (!mask) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (N <= 0 || H <= 0 || W <= 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (!geom_ok(g)) return fail(SBNET_EINVAL, "%s: bad geometry", who);
    if (pool != SBNET_POOL_MAX && pool != SBNET_POOL_AVG) return fail(SBNET_EINVAL, "%s: bad pool", who);
    if (mdt != SBNET_U8 && mdt != SBNET_F32) return fail(SBNET_EUNSUPPORTED, "%s: mask must be u8 or f32", who);
    if ((long long)N * g->bcount_h * g->bcount_w > 0x7fffffffLL || (long long)N * g->bcount_h > 0x7fffffffLL)
        return fail(SBNET_EUNSUPPORTED, "%s: more than 2^31 blocks", who);
    return SBNET_OK;
}

bool mask_flag_path(int N, const sbnet_geom *g) {
    return (long long)N * g->bcount_h * g->bcount_w <= kFlagPathMaxBlocks;
}

BlockDivs block_divs(const sbnet_geom *g) {
    BlockDivs dv;
    dv.per_sample = make_fastdiv((uint32_t)g->bcount_h * (uint32_t)g->bcount_w);
    dv.per_row = make_fastdiv((uint32_t)g->bcount_w);
    return dv;
}

// Pass 1 of the small-grid path: flags[blk] = 1 where block blk (lexicographic) is active, else 0, for all
// N * bcount_h * bcount_w blocks; flags must hold that many bytes rounded up to 16.
sbnet_status mask_to_flags(const char *who, const void *mask, sbnet_dtype mdt, int N, int H, int W,
                           const sbnet_geom *g, sbnet_pool pool, float threshold, uint8_t *flags, hipStream_t s) {
    sbnet_status st = check_mask_args(who, mask, mdt, N, H, W, g, pool);
    if (st != SBNET_OK) return st;
    if (!flags) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (!mask_flag_path(N, g)) return fail(SBNET_EUNSUPPORTED, "%s: more than %d blocks", who, kFlagPathMaxBlocks);
    const int total = N * g->bcount_h * g->bcount_w;
    const BlockDivs dv = block_divs(g);
    const double thr = (double)threshold;
    const dim3 grid((unsigned)((((total + 15) & ~15) + kRmThreads / 64 - 1) / (kRmThreads / 64)));   // one wave per flag byte, padding included
    const bool words = mdt == SBNET_U8 && (W % 4 == 0) && (((uintptr_t)mask) % 4 == 0);
    if (words) {
        // Smallest integer pool value v that counts as active: the decision everywhere is
        // (avg ? (double)v / area : (double)v) > (double)threshold, monotone in v, so it is a cutoff on v.
        const double area = (double)g->bsize_h * (double)g->bsize_w;
        const long long vmax = pool == SBNET_POOL_AVG ? 255LL * g->bsize_h * g->bsize_w : 255LL;
        auto active = [&](long long v) { return (pool == SBNET_POOL_AVG ? (double)v / area : (double)v) > thr; };
        long long lo = 0, hi = vmax + 1;                      // active(hi) taken as true: hi = "never"
        if (active(0)) hi = 0;
        while (hi - lo > 1) {                                 // invariant: !active(lo), hi active or vmax + 1
            const long long mid = lo + (hi - lo) / 2;
            if (active(mid)) hi = mid; else lo = mid;
        }
        if (hi <= 0x7fffffffLL) {
            int words_per_row = (g->bsize_w + 6) / 4, lp_shift = 0;           // most words a window row can touch
            while ((1 << lp_shift) < words_per_row && lp_shift < 6) ++lp_shift;
            if (pool == SBNET_POOL_MAX)
                hipLaunchKernelGGL((rm_pool_blocks_u8w<SBNET_POOL_MAX>), grid, dim3(kRmThreads), 0, s, (const uint32_t *)mask, H,
                                   W / 4, *g, dv, total, lp_shift, (int)hi, flags);
            else
                hipLaunchKernelGGL((rm_pool_blocks_u8w<SBNET_POOL_AVG>), grid, dim3(kRmThreads), 0, s, (const uint32_t *)mask, H,
                                   W / 4, *g, dv, total, lp_shift, (int)hi, flags);
            return launch_status(who);
        }
    }
#define SBNET_RM_BLOCKS(T, ACC, P, WORDS)                                                               \
    hipLaunchKernelGGL((rm_pool_blocks<T, ACC, P, WORDS>), grid, dim3(kRmThreads), 0, s, (const T *)mask, H, W, *g, \
                       dv, total, thr, flags)
    if (mdt == SBNET_U8) {
        if (pool == SBNET_POOL_MAX) { if (words) SBNET_RM_BLOCKS(uint8_t, int, SBNET_POOL_MAX, true); else SBNET_RM_BLOCKS(uint8_t, int, SBNET_POOL_MAX, false); }
        else { if (words) SBNET_RM_BLOCKS(uint8_t, int, SBNET_POOL_AVG, true); else SBNET_RM_BLOCKS(uint8_t, int, SBNET_POOL_AVG, false); }
    } else {
        if (pool == SBNET_POOL_MAX) SBNET_RM_BLOCKS(float, double, SBNET_POOL_MAX, false);
        else SBNET_RM_BLOCKS(float, double, SBNET_POOL_AVG, false);
    }
#undef SBNET_RM_BLOCKS
    return launch_status(who);
}

sbnet_status flags_to_indices(const char *who, const uint8_t *flags, int N, const sbnet_geom *g, int32_t *indices,
                              int32_t *count, int cap, hipStream_t s) {
    const int total = N * g->bcount_h * g->bcount_w;
    hipLaunchKernelGGL(rm_compact_flags, dim3((unsigned)((total + kRmThreads - 1) / kRmThreads)), dim3(kRmThreads), 0, s,
                       flags, total, *g, block_divs(g), indices, count, cap);
    return launch_status(who);
}

}  // namespace sbnet

extern "C" size_t sbnet_block_flags_bytes(int N, const sbnet_geom *g) {
    if (N <= 0 || !geom_ok(g)) return 0;
    return ((size_t)N * g->bcount_h * g->bcount_w + 15) & ~(size_t)15;
}

extern "C" sbnet_status sbnet_block_flags(const void *mask, sbnet_dtype mdt, int N, int H, int W, const sbnet_geom *g,
                                          sbnet_pool pool, float threshold, uint8_t *flags, size_t flags_bytes,
                                          void *stream) {
    if (N > 0 && geom_ok(g) && flags_bytes < sbnet_block_flags_bytes(N, g))
        return fail(SBNET_EINVAL, "sbnet_block_flags: flag buffer too small");
    return mask_to_flags("sbnet_block_flags", mask, mdt, N, H, W, g, pool, threshold, flags, (hipStream_t)stream);
}

// Argument checks and the two launches shared by both entry points; `workspace` is device memory of at
// least sbnet_workspace_bytes(N, g), every byte the kernels read from it is written by pass 1 first.
static sbnet_status reduce_mask_launch(const void *mask, sbnet_dtype mdt, int N, int H, int W,
                                       const sbnet_geom *g, sbnet_pool pool, float threshold,
                                       int32_t *indices, int32_t *count, int cap, void *workspace,
                                       size_t ws_bytes, void *stream) {
    if (!mask || !indices || !count || !workspace) return fail(SBNET_EINVAL, "sbnet_reduce_mask: null pointer");
    if (cap < 0) return fail(SBNET_EINVAL, "sbnet_reduce_mask: bad sizes");
    sbnet_status st = check_mask_args("sbnet_reduce_mask", mask, mdt, N, H, W, g, pool);
    if (st != SBNET_OK) return st;
    if (ws_bytes < sbnet_workspace_bytes(N, g)) return fail(SBNET_EINVAL, "sbnet_reduce_mask: workspace too small");
    hipStream_t s = (hipStream_t)stream;
    if (mask_flag_path(N, g)) {
        uint8_t *flags = (uint8_t *)workspace;
        st = mask_to_flags("sbnet_reduce_mask(pool)", mask, mdt, N, H, W, g, pool, threshold, flags, s);
        if (st != SBNET_OK) return st;
        return flags_to_indices("sbnet_reduce_mask(compact)", flags, N, g, indices, count, cap, s);
    }
    const int rows = N * g->bcount_h;
    const size_t acc_bytes = mdt == SBNET_U8 ? 4 : 8;
    const size_t lds = (size_t)W * acc_bytes;
    if (lds > 128 * 1024) return fail(SBNET_EUNSUPPORTED, "sbnet_reduce_mask: W too large for the column buffer");

    int32_t *rowcount = (int32_t *)workspace;
    uint8_t *flags = (uint8_t *)workspace + rowcount_bytes(rows);
    const double thr = (double)threshold;

    const bool vec4 = (W % 4 == 0) && (((uintptr_t)mask) % 16 == 0);
#define SBNET_RM_LAUNCH1(T, ACC, P, V)                                                                  \
    do {                                                                                                \
        if (lds > 48 * 1024)                                                                            \
            (void)hipFuncSetAttribute((const void *)rm_pool_rows<T, ACC, P, V>,                         \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);            \
        hipLaunchKernelGGL((rm_pool_rows<T, ACC, P, V>), dim3(rows), dim3(kRmThreads), lds, s,          \
                           (const T *)mask, H, W, *g, thr, rowcount, flags);                            \
    } while (0)
#define SBNET_RM_LAUNCH(T, ACC, P)                                                                      \
    do {                                                                                                \
        if (vec4) SBNET_RM_LAUNCH1(T, ACC, P, 4);                                                       \
        else SBNET_RM_LAUNCH1(T, ACC, P, 1);                                                            \
    } while (0)

    if (mdt == SBNET_U8) {
        if (pool == SBNET_POOL_MAX) SBNET_RM_LAUNCH(uint8_t, int, SBNET_POOL_MAX);
        else SBNET_RM_LAUNCH(uint8_t, int, SBNET_POOL_AVG);
    } else {
        if (pool == SBNET_POOL_MAX) SBNET_RM_LAUNCH(float, double, SBNET_POOL_MAX);
        else SBNET_RM_LAUNCH(float, double, SBNET_POOL_AVG);
    }
#undef SBNET_RM_LAUNCH
#undef SBNET_RM_LAUNCH1
    st = launch_status("sbnet_reduce_mask(pool)");
    if (st != SBNET_OK) return st;
    hipLaunchKernelGGL(rm_compact, dim3(rows), dim3(kRmThreads), 0, s, rowcount, flags, rows, g->bcount_h,
                       g->bcount_w, indices, count, cap);
    return launch_status("sbnet_reduce_mask(compact)");
}

extern "C" sbnet_status sbnet_reduce_mask(const void *mask, sbnet_dtype mdt, int N, int H, int W,
                                          const sbnet_geom *g, sbnet_pool pool, float threshold,
                                          int32_t *indices, int32_t *count, int cap, void *workspace,
                                          size_t ws_bytes, void *stream) {
    return reduce_mask_launch(mask, mdt, N, H, W, g, pool, threshold, indices, count, cap, workspace, ws_bytes,
                              stream);
}

// ---- the same call for callers that cannot hand over (or allocate) a workspace -------------------
// The row counts and flags live in a file-scope device array.  On the host the array's name is only a
// handle: its device address is looked up once per device with hipGetSymbolAddress and kept; kernels
// and every other host-side use take that address.
constexpr size_t kStaticScratchBytes = SBNET_REDUCE_MASK_STATIC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void *scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, 0 = not looked up

static sbnet_status static_scratch(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(SBNET_EHIP, "sbnet_reduce_mask_static: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(SBNET_EUNSUPPORTED, "sbnet_reduce_mask_static: device %d", dev);
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(SBNET_EHIP, "sbnet_reduce_mask_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return SBNET_OK;
}

extern "C" sbnet_status sbnet_reduce_mask_static(const void *mask, sbnet_dtype mdt, int N, int H, int W,
                                                 const sbnet_geom *g, sbnet_pool pool, float threshold,
                                                 int32_t *indices, int32_t *count, int cap, void *stream) {
    if (N <= 0 || !geom_ok(g)) return fail(SBNET_EINVAL, "sbnet_reduce_mask_static: bad sizes or geometry");
    const unsigned long long need = (unsigned long long)sbnet_workspace_bytes(N, g);
    if (need > kStaticScratchBytes)
        return fail(SBNET_EUNSUPPORTED, "sbnet_reduce_mask_static: %llu bytes of scratch needed for %d x %d x %d blocks, "
                    "the built-in buffer holds %llu; use sbnet_reduce_mask with a workspace",
                    need, N, g->bcount_h, g->bcount_w, (unsigned long long)kStaticScratchBytes);
    void *ws = nullptr;
    sbnet_status st = static_scratch(&ws);
    if (st != SBNET_OK) return st;
    return reduce_mask_launch(mask, mdt, N, H, W, g, pool, threshold, indices, count, cap, ws, kStaticScratchBytes,
                              stream);
}
