// Packed (logit, adapter index) keys of the wavefront top-k (Sec. 3.1: I(x) = top-k of G(x), ties to the
// lowest index): the maximum of the keys is the largest logit, and among equal logits the lowest index.
#pragma once
#include "common.hpp"

namespace meteora {

__device__ __forceinline__ uint64_t logit_key(float g, int index) {
    uint32_t u = __float_as_uint(g);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);   // monotonic map of finite floats to unsigned; -0 < +0 never ties with an index swap
    return ((uint64_t)u << 32) | (uint64_t)(0xffffffffu - (uint32_t)index);
}
__device__ __forceinline__ float key_logit(uint64_t key) {
    uint32_t u = (uint32_t)(key >> 32);
    u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
    return __uint_as_float(u);
}

}  // namespace meteora
