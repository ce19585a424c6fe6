// Element-wise add of two storage words as scatter-add defines it (Sec. 3.4 of arXiv 1801.02108, "Fused scatter-add
// kernel for residual blocks"): the sum is formed in fp32 and rounded to the storage type, round to nearest even.
// Shared by the NHWC and the transposing tile copies.
#pragma once
#include "common.h"

namespace sbnet {

template <int DT>
__device__ __forceinline__ uint32_t add_word(uint32_t y, uint32_t t);
template <>
__device__ __forceinline__ uint32_t add_word<SBNET_F32>(uint32_t y, uint32_t t) {
    return __float_as_uint(__uint_as_float(y) + __uint_as_float(t));
}
template <>
__device__ __forceinline__ uint32_t add_word<SBNET_BF16>(uint32_t y, uint32_t t) {
    const uint32_t lo = float_to_bf16_bits(bf16_bits_to_float(y & 0xffffu) + bf16_bits_to_float(t & 0xffffu));
    const uint32_t hi = float_to_bf16_bits(bf16_bits_to_float(y >> 16) + bf16_bits_to_float(t >> 16));
    return lo | (hi << 16);
}
__device__ __forceinline__ uint32_t f16_add_bits(uint32_t a, uint32_t b) {
    union { _Float16 h; uint16_t u; } x, y, r;
    x.u = (uint16_t)a; y.u = (uint16_t)b;
    r.h = (_Float16)((float)x.h + (float)y.h);
    return r.u;
}
template <>
__device__ __forceinline__ uint32_t add_word<SBNET_F16>(uint32_t y, uint32_t t) {
    return f16_add_bits(y & 0xffffu, t & 0xffffu) | (f16_add_bits(y >> 16, t >> 16) << 16);
}

}  // namespace sbnet
