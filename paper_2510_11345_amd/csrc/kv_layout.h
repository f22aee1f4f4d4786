// The two KV page layouts as device code, shared by the token writer and the fused decode step.
//   K page layout [page][h][d/8][kpos(t)][d%8]: 8 head-dim elements of a token are one 16-byte store.
//   V page layout [page][h][t/8][d][t%8]: they are 8 two-byte stores, 16 bytes apart.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace roll {

// kpos: inside blocks of min(P, 32) tokens, the low quad of every 8 tokens goes to the first half
// of the block and the high quad to the second half.
__device__ __forceinline__ int32_t k_slot(int32_t t, int32_t P) {
    const int32_t width = P < 32 ? P : 32;
    const int32_t u = t & (width - 1);
    return (t - u) + (u & 3) + 4 * (u >> 3) + (width >> 1) * ((u >> 2) & 1);
}

// Store 8 consecutive head-dim elements (slice c) of one token's K and V for head h.
// Hs: page stride in head blocks (the number of KV heads for dense pools).
__device__ __forceinline__ void store_kv_slice(uint4 kv, uint4 vv, uint4* __restrict__ k_pages,
                                               uint16_t* __restrict__ v_pages, int32_t page, int32_t t,
                                               int32_t h, int32_t c, int32_t P, int32_t Hs, int32_t D) {
    k_pages[(((int64_t)page * Hs + h) * (D / 8) + c) * P + k_slot(t, P)] = kv;
    uint16_t* vdst = v_pages + ((((int64_t)page * Hs + h) * (P / 8) + t / 8) * D + c * 8) * 8 + t % 8;
    const uint32_t w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        vdst[(2 * j) * 8] = (uint16_t)(w[j] & 0xFFFFu);
        vdst[(2 * j + 1) * 8] = (uint16_t)(w[j] >> 16);
    }
}

}  // namespace roll
