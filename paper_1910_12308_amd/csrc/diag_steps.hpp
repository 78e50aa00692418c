// H local SGD steps of a diagonal-quadratic objective on the two float4 a lane holds in its
// wave's 512-coordinate tile, in registers:
//   g = a (w - c) + sigma N(0, I),  w <- w - eta g,  a fresh Gaussian sample every step.
// One Philox call per step serves 8 consecutive coordinates (word p -> the Box-Muller pair of
// coordinates 8g+2p, 8g+2p+1), i.e. the float4 of two neighbouring lanes: the even lane draws for
// the group in the tile's first half, the odd lane for the one in the second half, and they swap
// the halves they do not need -- one generator call per lane and step for 8 normals.
#pragma once
#include "gossip_common.hpp"

namespace swarm {

#if defined(__HIPCC__)
// Two normals of standard deviation sigma from one word: u1 = (low half + 1/2) 2^-16 in (0,1),
// u2 = high half * 2^-16 in [0,1); (r cos 2 pi u2, r sin 2 pi u2), r = sigma sqrt(-2 ln u1), with
// sigma^2 folded into the factor of the logarithm: scale = -2 ln 2 sigma^2.  Hardware log2 / sqrt /
// sine / cosine (the latter two take revolutions, so u2 needs no range reduction).
__device__ __forceinline__ void box_muller16(uint32_t w, float scale, float &n0, float &n1) {
    const float u1 = fmaf((float)(w & 0xFFFFu), 0x1p-16f, 0x1p-17f);
    const float u2 = (float)(w >> 16) * 0x1p-16f;
    const float r = __builtin_amdgcn_sqrtf(scale * __builtin_amdgcn_logf(u1));
    n0 = r * __builtin_amdgcn_cosf(u2);
    n1 = r * __builtin_amdgcn_sinf(u2);
}
#endif

__device__ __forceinline__ f4 diag_update(f4 w, const f4 a, const f4 c, const f4 noise, float lr) {
    const f4 t = w - c;
    f4 g;
    g.x = fmaf(a.x, t.x, noise.x); g.y = fmaf(a.y, t.y, noise.y);
    g.z = fmaf(a.z, t.z, noise.z); g.w = fmaf(a.w, t.w, noise.w);
    w.x = fmaf(-lr, g.x, w.x); w.y = fmaf(-lr, g.y, w.y);
    w.z = fmaf(-lr, g.z, w.z); w.w = fmaf(-lr, g.w, w.w);
    return w;
}

// wA / wB: the lane's float4 number `lane` and `lane + 64` of tile `tile` of the node's row.
// Every lane of the wave must call this (the neighbour swap is a cross-lane move).
template <bool NOISE>
__device__ __forceinline__ void diag_steps(f4 &wA, f4 &wB, const f4 aA, const f4 aB, const f4 cA, const f4 cB,
                                           uint32_t node, uint64_t tile, uint32_t lane, uint32_t H, float lr,
                                           float sigma, uint64_t seed, uint32_t event) {
    const bool odd = lane & 1u;
    const uint64_t group = tile * (TILE / 8) + (lane >> 1) + (odd ? 32u : 0u);
    const float scale = -1.3862943611198906f * sigma * sigma;     // -2 ln 2 sigma^2
    for (uint32_t q = 0; q < H; ++q) {
        f4 nA = {0.f, 0.f, 0.f, 0.f}, nB = nA;
        if (NOISE) {
            const Words4 w = stream(seed, TAG_NOISE, q, node, event, group);
            // even lane: words 0,1 of its own call (first half) and of the neighbour's (second half);
            // odd lane: words 2,3 of the neighbour's call (first half) and of its own (second half).
            const uint32_t r0 = swap_with_neighbour(odd ? w.w0 : w.w2);
            const uint32_t r1 = swap_with_neighbour(odd ? w.w1 : w.w3);
            float z0, z1, z2, z3, z4, z5, z6, z7;
            box_muller16(odd ? r0 : w.w0, scale, z0, z1);
            box_muller16(odd ? r1 : w.w1, scale, z2, z3);
            box_muller16(odd ? w.w2 : r0, scale, z4, z5);
            box_muller16(odd ? w.w3 : r1, scale, z6, z7);
            nA = f4{z0, z1, z2, z3};
            nB = f4{z4, z5, z6, z7};
        }
        wA = diag_update(wA, aA, cA, nA, lr);
        wB = diag_update(wB, aB, cB, nB, lr);
    }
}

}  // namespace swarm
