// Types shared by the convolution kernels (conv.hip: generic direct + MFMA kernels;
// conv16.hip: the register-stationary 3x3 kernel for 16-pixel-wide output tiles;
// conv3.hip: the LDS-tiled 3x3 kernel for any stride and tile).
#pragma once
#include "common.h"

namespace sbnet {

// ------------------------------------------------------------------------------------------
// element helpers
// ------------------------------------------------------------------------------------------
template <int DT> struct Elem;
template <> struct Elem<SBNET_F32> {
    typedef float T;
    static __device__ __forceinline__ float load(const T *p) { return *p; }
    static __device__ __forceinline__ void store(T *p, float v) { *p = v; }
};
template <> struct Elem<SBNET_BF16> {
    typedef uint16_t T;
    static __device__ __forceinline__ float load(const T *p) { return bf16_bits_to_float(*p); }
    static __device__ __forceinline__ void store(T *p, float v) { *p = (uint16_t)float_to_bf16_bits(v); }
};
template <> struct Elem<SBNET_F16> {
    typedef _Float16 T;
    static __device__ __forceinline__ float load(const T *p) { return (float)*p; }
    static __device__ __forceinline__ void store(T *p, float v) { *p = (_Float16)v; }
};

struct ConvParams {
    const void *in;          // tile stack [cap][th][tw][Cin]   or feature map [N][H][W][Cin]
    void *out;               // tile stack [cap][oh][ow][Cout]  or feature map [N][Ho][Wo][Cout]
    const void *w;           // packed weights
    size_t w32_offset;       // MFMA path: start (in 16-byte units) of the 32x32x16 operand copy inside w
    const float *bias;       // [Cout] or null
    const int32_t *indices;  // fused form only
    const int32_t *count;
    int cap;
    int th, tw, oh, ow;
    int Cin, Cout;
    int kh, kw, sh, sw;
    int relu, add;
    sbnet_geom g_in, g_out;  // fused form only
    int H, W, Ho, Wo;        // fused form only
    // fused form fed by block flags instead of an index list (conv16.hip): the kernel compacts the flags of all
    // total_blocks blocks itself and also writes the list and the count it derives for later consumers
    const uint8_t *flags;    // [total_blocks] padded to 16 bytes, or null
    int total_blocks;
    int32_t *indices_out;    // [cap][3]
    int32_t *count_out;      // [1]
    FastDiv div_bps, div_bw, div_grid;       // blocks per sample, blocks per block row, workgroups along x
    int small_cost8;         // conv3.hip, two tile shapes in one launch: cost of the smaller item in eighths of the larger
    int wide_min_items;      // conv3.hip, 64-channel or wider output groups in one launch: wide from this many work items
    // MFMA path work decomposition
    int CinP;                // Cin rounded up to 32
    int CC;                  // channels per LDS chunk (multiple of 32)
    int nchunks;
    int mpasses;             // passes of 256 output pixels per tile
    int ngroups;             // groups of 64 output channels
    int lds_rows;            // input rows held in LDS per pass (upper bound)
    FastDiv div_ow, div_tw, div_cv, div_cv_last, div_pn, div_ng;
};


typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

template <int DT>
__device__ __forceinline__ f32x4 mfma16x16x32(uint4 a, uint4 b, f32x4 c) {
    if (DT == SBNET_BF16) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two fp32 -> two storage elements in one word (round to nearest even; bf16 uses gfx950's
// packed hardware conversion)
template <int DT>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    if (DT == SBNET_BF16) {
        const f32x2_t f = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
    }
    union { _Float16 h[2]; uint32_t u; } v;
    v.h[0] = (_Float16)lo;
    v.h[1] = (_Float16)hi;
    return v.u;
}
template <int DT>
__device__ __forceinline__ float unpack_lo(uint32_t w) {
    if (DT == SBNET_BF16) return bf16_bits_to_float(w & 0xffffu);
    union { _Float16 h[2]; uint32_t u; } v;
    v.u = w;
    return (float)v.h[0];
}
template <int DT>
__device__ __forceinline__ float unpack_hi(uint32_t w) {
    if (DT == SBNET_BF16) return bf16_bits_to_float(w >> 16);
    union { _Float16 h[2]; uint32_t u; } v;
    v.u = w;
    return (float)v.h[1];
}

// ------------------------------------------------------------------------------------------
// shared by the 32x32x16 MFMA kernels (conv16.hip, conv3.hip)
// ------------------------------------------------------------------------------------------
constexpr uint32_t kBufWord3 = 0x00020000u;      // raw buffer descriptor, 32-bit data format
constexpr uint32_t kOutOfRange = 0x80000000u;    // offset beyond any descriptor these kernels build (all below 2 GiB)

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

template <int DT>
__device__ __forceinline__ f32x16 mfma32x32x16(uint4 a, uint4 b, f32x16 c) {
    if (DT == SBNET_BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
}

typedef short i16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t relu_pair(uint32_t w, uint32_t floor2) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(i16x2, w), __builtin_bit_cast(i16x2, floor2)));
}
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t off) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void buf_store16(__amdgpu_buffer_rsrc_t r, uint32_t off, uint4 d) {
    u32x4 v;
    v[0] = d.x; v[1] = d.y; v[2] = d.z; v[3] = d.w;
    // non-temporal: the results are not read again here and should not push input lines, which neighbouring
    // tiles read again for their halos, out of L2
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)off, 0, 2);
}

// conv16.hip: returns true when it took the job (status in *st), false when the shape is not its own.
// With p.flags set it only takes shapes its flag-fed variant serves (16 x 16 output blocks, at most 65 536 blocks).
bool conv16_try(sbnet_dtype dt, bool fused, const ConvParams &p, hipStream_t s, sbnet_status *st, const char *who);
// the same decision without a launch (p.oh, p.ow set)
bool conv16_accepts(sbnet_dtype dt, bool fused, const ConvParams &p);
// conv3.hip: the same contract for the LDS-tiled 3x3 kernel (any stride, tile size and channel counts that are multiples of 8).
bool conv3_try(sbnet_dtype dt, bool fused, const ConvParams &p, hipStream_t s, sbnet_status *st, const char *who);

}  // namespace sbnet
