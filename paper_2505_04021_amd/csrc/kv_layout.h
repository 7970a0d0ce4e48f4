// Where an element of a K or V tile sits inside a block (gfx950 operand order).
//
// A block holds, per kv head, the K tile followed by the V tile, T = 16 tokens each;
// e4m3 blocks start with a 128-byte header (fp32 sK[Hkv], fp32 sV[Hkv]).  Tiles are stored
// in the lane order of the MFMA operands the attention kernels feed them to:
//   bf16 K: 16-byte unit (c, t)      = K[t][8c .. 8c+7]                  at ((c*16)+t)*16
//   bf16 V: 16-byte unit (jp, G, dl) = V[4G..4G+3][32jp+dl] ,
//                                      V[4G..4G+3][32jp+16+dl]           at ((jp*4+G)*16+dl)*16
//   e4m3 K: 16-byte unit (j2, G, t)  = K[t][8(8j2+G)+0..7] , K[t][8(8j2+4+G)+0..7]
//   e4m3 V: 16-byte unit (jq, G, dl) = V[4G..4G+3][64jq+16u+dl], u = 0..3
// The functions return the offset in elements from the start of the tile.
#pragma once
#include "pkv_internal.h"

constexpr int PKV_T = 16;   // tokens per block the kernels are built for

template <int DT>
__device__ __forceinline__ size_t k_elem_off(int t, int dd) {
    if (DT == PKV_BF16) return ((size_t)((dd >> 3) * 16 + t)) * 8 + (dd & 7);
    const int c8 = dd >> 3, j = c8 >> 2, Gk = c8 & 3, j2 = j >> 1, hf = j & 1;
    return ((size_t)((j2 * 4 + Gk) * 16 + t)) * 16 + hf * 8 + (dd & 7);
}

template <int DT>
__device__ __forceinline__ size_t v_elem_off(int t, int dd) {
    const int G = t >> 2, e = t & 3;
    if (DT == PKV_BF16) {
        const int jp = dd >> 5, half = (dd >> 4) & 1, dl = dd & 15;
        return ((size_t)((jp * 4 + G) * 16 + dl)) * 8 + half * 4 + e;
    }
    const int jq = dd >> 6, u = (dd >> 4) & 3, dl = dd & 15;
    return ((size_t)((jq * 4 + G) * 16 + dl)) * 16 + u * 4 + e;
}

// start of a block in the pool
__device__ __forceinline__ uint8_t *block_ptr(const AttnDesc &d, uint32_t id) {
    const uint32_t f = fastdiv_div(id, d.slots_div);
    const uint32_t s = id - f * d.slots_div.d;
    return const_cast<uint8_t *>(d.pool_base) + (uint64_t)f * d.frame_bytes + (uint64_t)s * d.block_bytes;
}
