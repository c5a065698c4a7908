// Where the matrix-core kernel keeps a row in LDS and which lane reads which position: shared by the
// kernel (perq_mfma.hip) and by the host routine that arranges a permutation for its gather
// (perq_perm_arrange in perq_host.cpp).
#pragma once
#include <cstdint>

namespace perq {
namespace layout {

// 16-byte granule -> slot inside a staged row (an involution: bits 4..6 select the xor pattern
// for bits 0..2)
__host__ __device__ inline __attribute__((always_inline)) uint32_t granule_slot(uint32_t g) {
    const uint32_t c = (g >> 4) & 7u;
    return g ^ (((c & 3u) << 1) | (c >> 2));
}

// byte offset of channel a inside its staged row
__host__ __device__ inline __attribute__((always_inline)) uint32_t channel_offset(uint32_t a) {
    return (granule_slot(a >> 3) << 4) | ((a & 7u) << 1);
}

// high-K mode (b >= 1024): position inside the tile of row m (5 bits), contraction index K (7 bits)
__host__ __device__ inline __attribute__((always_inline)) uint32_t hk_pos(uint32_t m, uint32_t K) {
    return (m & 15u) | (K << 4) | ((m >> 4) << 11);
}

// row of the +-1 operand that lane l (0..31) of a half-wave holds
__host__ __device__ inline __attribute__((always_inline)) uint32_t lane_sigma(uint32_t l) {
    return 16u * ((l >> 2) & 1u) + 4u * (l >> 3) + (l & 3u);
}

// Position inside a 4096-wide tile of element e (0..7) of operand fragment f (0..7) in lane
// l (0..31) of half-wave h: read instruction (f, e) of the element-wise gather.
__host__ __device__ inline __attribute__((always_inline)) uint32_t gather_pos(bool high_k, uint32_t l, uint32_t h, uint32_t f, uint32_t e) {
    return high_k ? hk_pos(lane_sigma(l), 16u * f + 8u * h + e)
                  : (l * 4u + (f >> 1)) * 32u + 16u * (f & 1u) + 8u * h + e;
}

// Rows this wide are staged in the placement a caller prepared for the permutation
// (perq_perm_prepare); narrower ones keep granule_slot.
__host__ __device__ inline __attribute__((always_inline)) bool placement_applies(int32_t d) { return d > 8192; }

}  // namespace layout
}  // namespace perq
