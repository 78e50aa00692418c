// One wave's 512-coordinate tile of one step of Algorithm 1 (see interact.hip), shared by the
// interaction kernel and by the kernel that runs a least-squares initiator's local steps and its
// interaction in one workgroup.
#pragma once
#include "diag_steps.hpp"
#include "gossip_common.hpp"
#include "objectives.h"

namespace swarm {

struct InteractArgs {
    GossipArgs g;
    const SeqDesc *descs;     // device: one per grid row, or null: the single interaction `one`
    SeqDesc one;
    const float *A, *C;       // n x d objective data (LOCAL only)
    float sigma, lr;
};

// LOCAL: 0 = the pending update is W_i - Xhat_i where the descriptor says so; 1 / 2 = local steps of the
// diagonal objective in registers, with / without gradient noise; 3 = the pending update of the lane's two
// float4 is handed in (givenA, givenB).
template <int BITS, int LOCAL>
__device__ __forceinline__ void interact_tile(const InteractArgs &ia, const SeqDesc sd, uint64_t tile, uint32_t lane,
                                              f4 givenA = f4{0.f, 0.f, 0.f, 0.f}, f4 givenB = f4{0.f, 0.f, 0.f, 0.f}) {
    const GossipArgs &a = ia.g;
    const uint32_t ni = sd.ni, nj = sd.nj, event = sd.event;
    const uint64_t kA = tile * TILE + 4ull * lane, kB = kA + TILE / 2;
    const bool inA = kA < a.d, inB = kB < a.d;
    const uint64_t lA = inA ? kA : a.d - 4, lB = inB ? kB : a.d - 4;   // past the row end: re-read its last float4
    const uint64_t oi = (uint64_t)ni * a.d, oj = (uint64_t)nj * a.d;
    float *xi = a.X + oi, *xj = a.X + oj, *hi = a.Xhat + oi;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const f4 xiA = ldg_nt(xi + lA), xiB = ldg_nt(xi + lB);
    const f4 xjA = ldg_nt(xj + lA), xjB = ldg_nt(xj + lB);
    f4 dA = zero, dB = zero;
    if (LOCAL == 3) {
        dA = givenA;
        dB = givenB;
    } else if (LOCAL) {
        const f4 hA = ldg_nt(hi + lA), hB = ldg_nt(hi + lB);
        const f4 aA = ldg_nt(ia.A + oi + lA), aB = ldg_nt(ia.A + oi + lB);
        const f4 cA = ldg_nt(ia.C + oi + lA), cB = ldg_nt(ia.C + oi + lB);
        f4 wA = hA, wB = hB;
        diag_steps<LOCAL == 1>(wA, wB, aA, aB, cA, cB, ni, tile, lane, (sd.flags >> 8) & 0xFFu, ia.lr, ia.sigma, a.seed, event);
        dA = wA - hA;
        dB = wB - hB;
    } else if (sd.flags & SEQ_HAS_DELTA) {
        const float *wi = a.W + oi;
        dA = ldg_nt(wi + lA) - ldg_nt(hi + lA);
        dB = ldg_nt(wi + lB) - ldg_nt(hi + lB);
    }
    f4 avgA, avgB;
    if constexpr (BITS > 0) {
        const LaneRandom ri = row_random(a.seed, ni, event, tile, lane);
        const LaneRandom rj = row_random(a.seed, nj, event, tile, lane);
        bool clampedA = false, clampedB = false;
        int failsA = 0, failsB = 0;
        int ziA[4], ziB[4], zjA[4], zjB[4];
        const uint64_t ciA = round_float4<BITS>(xiA, ri.a0, ri.a1, a.inv_eps, ziA, clampedA);
        const uint64_t ciB = round_float4<BITS>(xiB, ri.b0, ri.b1, a.inv_eps, ziB, clampedB);
        const uint64_t cjA = round_float4<BITS>(xjA, rj.a0, rj.a1, a.inv_eps, zjA, clampedA);
        const uint64_t cjB = round_float4<BITS>(xjB, rj.b0, rj.b1, a.inv_eps, zjB, clampedB);
        const float half_eps = 0.5f * a.eps;
        avgA = averaged<BITS>(ziA, cjA, xiA, zero, a.inv_eps, half_eps, zjA, failsA, clampedA);
        avgB = averaged<BITS>(ziB, cjB, xiB, zero, a.inv_eps, half_eps, zjB, failsB, clampedB);
        uint8_t *pub_i = a.ring + ni * a.row_bytes, *pub_j = a.ring + nj * a.row_bytes;
        if (inA) { store_code<BITS>(pub_i, kA / 4, ciA); store_code<BITS>(pub_j, kA / 4, cjA); }
        if (inB) { store_code<BITS>(pub_i, kB / 4, ciB); store_code<BITS>(pub_j, kB / 4, cjB); }
        report(a.counters, (inA ? failsA : 0) + (inB ? failsB : 0), (inA && clampedA) || (inB && clampedB));
    } else {
        avgA = 0.5f * (xiA + xjA);
        avgB = 0.5f * (xiB + xjB);
    }
    if (inA) { const f4 o = avgA + dA; stg_nt(xi + kA, o); stg_nt(hi + kA, o); stg_nt(xj + kA, avgA); }
    if (inB) { const f4 o = avgB + dB; stg_nt(xi + kB, o); stg_nt(hi + kB, o); stg_nt(xj + kB, avgB); }
}

}  // namespace swarm
