// reduce_mask: binary computation mask -> ordered list of active blocks
// (Sec. 3.1 "Reduce mask to indices" and Sec. 3.4 "Fused downsample and indexing kernel" of
// arXiv 1801.02108).
//
// The paper appends indices with a global atomic counter, which gives an arbitrary order.
// Here the list is produced in lexicographic (n, by, bx) order without atomics:
//   pass 1  one workgroup per block row: coalesced column pooling of the window rows into LDS
//           (four columns per thread and all rows of a window in flight, so the window costs one
//           memory latency),
//           then one thread per block pools its window columns, thresholds, stores a flag byte
//           and the row's number of active blocks;
//   pass 2  one workgroup per block row: exclusive prefix over the row counts, then wavefront
//           ballot + popcount compaction of the row's flags into the index list.
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

}  // namespace sbnet

using namespace sbnet;

static size_t rowcount_bytes(int rows) { return (((size_t)rows * 4) + 15) & ~(size_t)15; }

extern "C" size_t sbnet_workspace_bytes(int N, const sbnet_geom *g) {
    if (N <= 0 || !geom_ok(g)) return 0;
    const size_t rows = (size_t)N * g->bcount_h;
    return rowcount_bytes((int)rows) + ((rows * g->bcount_w + 15) & ~(size_t)15);
}

// Argument checks and the two launches shared by both entry points; `workspace` is device memory of at
// least sbnet_workspace_bytes(N, g), every byte the kernels read from it is written by pass 1 first.
static sbnet_status reduce_mask_launch(const void *mask, sbnet_dtype mdt, int N, int H, int W,
                                       const sbnet_geom *g, sbnet_pool pool, float threshold,
                                       int32_t *indices, int32_t *count, int cap, void *workspace,
                                       size_t ws_bytes, void *stream) {
    if (!mask || !indices || !count || !workspace) return fail(SBNET_EINVAL, "sbnet_reduce_mask: null pointer");
    if (N <= 0 || H <= 0 || W <= 0 || cap < 0) return fail(SBNET_EINVAL, "sbnet_reduce_mask: bad sizes");
    if (!geom_ok(g)) return fail(SBNET_EINVAL, "sbnet_reduce_mask: bad geometry");
    if (pool != SBNET_POOL_MAX && pool != SBNET_POOL_AVG) return fail(SBNET_EINVAL, "sbnet_reduce_mask: bad pool");
    if (mdt != SBNET_U8 && mdt != SBNET_F32)
        return fail(SBNET_EUNSUPPORTED, "sbnet_reduce_mask: mask must be u8 or f32");
    if (ws_bytes < sbnet_workspace_bytes(N, g)) return fail(SBNET_EINVAL, "sbnet_reduce_mask: workspace too small");
    const long long rows_ll = (long long)N * g->bcount_h;
    if (rows_ll * g->bcount_w > 0x7fffffffLL || rows_ll > 0x7fffffffLL)
        return fail(SBNET_EUNSUPPORTED, "sbnet_reduce_mask: more than 2^31 blocks");
    const int rows = (int)rows_ll;
    const size_t acc_bytes = mdt == SBNET_U8 ? 4 : 8;
    const size_t lds = (size_t)W * acc_bytes;
    if (lds > 128 * 1024) return fail(SBNET_EUNSUPPORTED, "sbnet_reduce_mask: W too large for the column buffer");

    int32_t *rowcount = (int32_t *)workspace;
    uint8_t *flags = (uint8_t *)workspace + rowcount_bytes(rows);
    hipStream_t s = (hipStream_t)stream;
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
    sbnet_status st = launch_status("sbnet_reduce_mask(pool)");
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
