// Philox4x32-10 and the named random streams of the swarm simulation (gfx950).
// The paper only asks for unbiased rounding (Corollary 2.1, item 1) and i.i.d.
// sampling; a counter-based generator lets every thread draw its numbers from
// (seed, stream tag, local-step index, node or edge id, event id, index) alone.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swarm {

enum : uint32_t { TAG_SR = 1, TAG_NOISE = 2, TAG_MATCH = 3, TAG_PICK = 4, TAG_BATCH = 5,
                  TAG_STALE = 6, TAG_DATA = 7, TAG_LABEL = 8, TAG_STEPS = 9 };

struct Words4 { uint32_t w0, w1, w2, w3; };

__host__ __device__ __forceinline__ Words4 philox4x32_10(uint32_t k0, uint32_t k1, uint32_t c0,
                                                         uint32_t c1, uint32_t c2, uint32_t c3) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c0 = n0; c1 = (uint32_t)p1; c2 = n2; c3 = (uint32_t)p0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return Words4{c0, c1, c2, c3};
}

// Counter layout: c0 = index low 32 bits, c1 = tag<<24 | q<<16 | index bits 32..47,
// c2 = node / edge id, c3 = event (round or interaction number).
__host__ __device__ __forceinline__ Words4 stream(uint64_t seed, uint32_t tag, uint32_t q,
                                                  uint32_t ident, uint32_t event, uint64_t index) {
    return philox4x32_10((uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)index,
                         (tag << 24) | ((q & 0xFFu) << 16) | (uint32_t)((index >> 32) & 0xFFFFu),
                         ident, event);
}

// floor(u * m) for u = word / 2^32.
__host__ __device__ __forceinline__ uint32_t scaled_index(uint32_t word, uint32_t m) {
    return (uint32_t)(((uint64_t)word * m) >> 32);
}

#if defined(__HIPCC__)
// Two standard normals from two words (Box-Muller): u1 = ((wa>>8)+1) 2^-24 in (0,1],
// u2 = (wb>>8) 2^-24 in [0,1); (r cos 2 pi u2, r sin 2 pi u2), r = sqrt(-2 ln u1).
// Uses the hardware transcendentals directly: log2 and sqrt are accurate to 1 ulp, and sine /
// cosine take their argument in revolutions, so u2 needs no range reduction.  Measured against
// float64 over 4 M draws including u1 -> 0, u1 -> 1 and the quadrant boundaries of u2:
// |error| <= 3.3e-7 max(1, |z|), the same order as the library routines (2.2e-7).
__device__ __forceinline__ void box_muller(uint32_t wa, uint32_t wb, float &n0, float &n1) {
    const float u1 = (float)((wa >> 8) + 1u) * 0x1p-24f;
    const float u2 = (float)(wb >> 8) * 0x1p-24f;
    const float r = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(u1));   // -2 ln 2 * log2 u1
    n0 = r * __builtin_amdgcn_cosf(u2);
    n1 = r * __builtin_amdgcn_sinf(u2);
}
#endif

}  // namespace swarm
