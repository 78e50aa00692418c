// Whole round in one pass for per-coordinate objectives (diagonal quadratics): the H local
// steps of both nodes of a pair are taken in registers and fed straight into the quantized
// gossip step, so the live copy W never travels through memory.  Same arithmetic, in the
// same order, as local_diag_kernel followed by gossip_pairs_kernel; per pair-coordinate it
// reads X_i, X_j, a_i, a_j, c_i, c_j (24 B) and the two partner codes, and writes X_i', X_j'
// (8 B) and the two published codes.
//   deferred apply:  z = SR(X),  X' = eps (z_i + z_j')/2 + (w - X)      (the paper's rule)
//   in-place apply:  z = SR(w),  X' = eps (z_i + z_j')/2, decoded against w
#include "diag_steps.hpp"
#include "gossip_common.hpp"
#include "objectives.h"

namespace swarm {

#ifndef SWARM_FUSED_WAVES
#define SWARM_FUSED_WAVES 8
#endif
constexpr int FWAVES = SWARM_FUSED_WAVES;     // waves per workgroup of the one-pass kernels

struct FusedArgs {
    GossipArgs g;
    const float *A, *C;       // n x d objective data
    float sigma, lr;
};

template <int BITS, int STALE, bool INPLACE, bool NOISE, bool FULL>
__device__ __forceinline__ void fused_pair_tile(const FusedArgs &fa, const PairDesc pd, uint64_t tile, uint32_t lane) {
    const GossipArgs &a = fa.g;
    const uint64_t kA = tile * TILE + 4ull * lane, kB = kA + TILE / 2;
    const bool inA = FULL || kA < a.d, inB = FULL || kB < a.d;
    const uint64_t lA = inA ? kA : a.d - 4, lB = inB ? kB : a.d - 4;   // past the row end: re-read its last float4
    const uint32_t ni = pd.ni, nj = pd.nj;
    const uint64_t oi = (uint64_t)ni * a.d, oj = (uint64_t)nj * a.d;
    float *xi = a.X + oi, *xj = a.X + oj;
    const uint32_t si = STALE == 0 ? 0u : (pd.flags & 0xFFu), sj = STALE == 0 ? 0u : ((pd.flags >> 8) & 0xFFu);
    const bool stale_i = STALE == 1 || STALE == 3 || (STALE == 2 && si != 0);
    const bool stale_j = STALE == 1 || (STALE == 2 && sj != 0);

    const f4 xiA = ldg_nt(xi + lA), xjA = ldg_nt(xj + lA), xiB = ldg_nt(xi + lB), xjB = ldg_nt(xj + lB);
    const f4 aiA = ldg_nt(fa.A + oi + lA), ajA = ldg_nt(fa.A + oj + lA), aiB = ldg_nt(fa.A + oi + lB), ajB = ldg_nt(fa.A + oj + lB);
    const f4 ciA_ = ldg_nt(fa.C + oi + lA), cjA_ = ldg_nt(fa.C + oj + lA), ciB_ = ldg_nt(fa.C + oi + lB), cjB_ = ldg_nt(fa.C + oj + lB);

    const uint64_t slot_bytes = (uint64_t)a.n * a.row_bytes;
    uint8_t *pub_i = a.ring + a.slot_now * slot_bytes + ni * a.row_bytes;
    uint8_t *pub_j = a.ring + a.slot_now * slot_bytes + nj * a.row_bytes;
    uint64_t seenjA = 0, seenjB = 0, seeniA = 0, seeniB = 0;
    if (stale_i) {
        const uint8_t *src = a.ring + ((a.slot_now + a.ring_depth - si) % a.ring_depth) * slot_bytes + nj * a.row_bytes;
        seenjA = load_code<BITS>(src, lA / 4);
        seenjB = load_code<BITS>(src, lB / 4);
    }
    if (stale_j) {
        const uint8_t *src = a.ring + ((a.slot_now + a.ring_depth - sj) % a.ring_depth) * slot_bytes + ni * a.row_bytes;
        seeniA = load_code<BITS>(src, lA / 4);
        seeniB = load_code<BITS>(src, lB / 4);
    }

    // local steps of both nodes on this lane's four float4 (step counts travel in the descriptor)
    const uint32_t Hi = pd.steps & 0xFFu, Hj = (pd.steps >> 8) & 0xFFu;
    f4 wiA = xiA, wiB = xiB, wjA = xjA, wjB = xjB;
    diag_steps<NOISE>(wiA, wiB, aiA, aiB, ciA_, ciB_, ni, tile, lane, Hi, fa.lr, fa.sigma, a.seed, a.event);
    diag_steps<NOISE>(wjA, wjB, ajA, ajB, cjA_, cjB_, nj, tile, lane, Hj, fa.lr, fa.sigma, a.seed, a.event);
    // what is quantized / used as decoding key, and what is added to the average
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const f4 qiA = INPLACE ? wiA : xiA, qiB = INPLACE ? wiB : xiB, qjA = INPLACE ? wjA : xjA, qjB = INPLACE ? wjB : xjB;
    const f4 diA = INPLACE ? zero : wiA - xiA, diB = INPLACE ? zero : wiB - xiB;
    const f4 djA = INPLACE ? zero : wjA - xjA, djB = INPLACE ? zero : wjB - xjB;

    const LaneRandom ri = row_random(a.seed, ni, a.event, tile, lane);
    const LaneRandom rj = row_random(a.seed, nj, a.event, tile, lane);
    bool clampedA = false, clampedB = false;
    int failsA = 0, failsB = 0;
    int ziA[4], ziB[4], zjA[4], zjB[4];
    const ReadScale rsi = read_scale(a, si, a.eps, a.inv_eps), rsj = read_scale(a, sj, a.eps, a.inv_eps);
    const float inv_now = rsi.inv_now;
    const uint64_t ciA = round_float4<BITS>(qiA, ri.a0, ri.a1, inv_now, ziA, clampedA);
    const uint64_t ciB = round_float4<BITS>(qiB, ri.b0, ri.b1, inv_now, ziB, clampedB);
    const uint64_t cjA = round_float4<BITS>(qjA, rj.a0, rj.a1, inv_now, zjA, clampedA);
    const uint64_t cjB = round_float4<BITS>(qjB, rj.b0, rj.b1, inv_now, zjB, clampedB);
    f4 oiA, oiB, ojA, ojB;
    if (a.eps_slots) {                           // one scale per round: the partner's code may be on an older lattice
        float far = 0.f;
        oiA = averaged_mixed<BITS>(ziA, stale_i ? seenjA : cjA, qiA, diA, rsi.eps_now, rsi.eps_old, rsi.inv_old,
                                   stale_i ? nullptr : zjA, failsA, clampedA, far, inA);
        oiB = averaged_mixed<BITS>(ziB, stale_i ? seenjB : cjB, qiB, diB, rsi.eps_now, rsi.eps_old, rsi.inv_old,
                                   stale_i ? nullptr : zjB, failsB, clampedB, far, inB);
        ojA = averaged_mixed<BITS>(zjA, stale_j ? seeniA : ciA, qjA, djA, rsj.eps_now, rsj.eps_old, rsj.inv_old,
                                   stale_j ? nullptr : ziA, failsA, clampedA, far, inA);
        ojB = averaged_mixed<BITS>(zjB, stale_j ? seeniB : ciB, qjB, djB, rsj.eps_now, rsj.eps_old, rsj.inv_old,
                                   stale_j ? nullptr : ziB, failsB, clampedB, far, inB);
        report_far(a.far_bits, far);
    } else {
        const float half_eps = 0.5f * rsi.eps_now;
        oiA = averaged<BITS>(ziA, stale_i ? seenjA : cjA, qiA, diA, inv_now, half_eps, stale_i ? nullptr : zjA, failsA, clampedA);
        oiB = averaged<BITS>(ziB, stale_i ? seenjB : cjB, qiB, diB, inv_now, half_eps, stale_i ? nullptr : zjB, failsB, clampedB);
        ojA = averaged<BITS>(zjA, stale_j ? seeniA : ciA, qjA, djA, inv_now, half_eps, stale_j ? nullptr : ziA, failsA, clampedA);
        ojB = averaged<BITS>(zjB, stale_j ? seeniB : ciB, qjB, djB, inv_now, half_eps, stale_j ? nullptr : ziB, failsB, clampedB);
    }
    if (inA) {
        stg_nt(xi + kA, oiA); stg_nt(xj + kA, ojA);
        store_code<BITS>(pub_i, kA / 4, ciA); store_code<BITS>(pub_j, kA / 4, cjA);
    }
    if (inB) {
        stg_nt(xi + kB, oiB); stg_nt(xj + kB, ojB);
        store_code<BITS>(pub_i, kB / 4, ciB); store_code<BITS>(pub_j, kB / 4, cjB);
    }
    report(a.counters, (inA ? failsA : 0) + (inB ? failsB : 0), (inA && clampedA) || (inB && clampedB));
}

template <int BITS, int STALE, bool INPLACE, bool NOISE>
__global__ __launch_bounds__(FWAVES * 64) void fused_pairs_kernel(const FusedArgs fa) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = (uint64_t)blockIdx.x * FWAVES + (threadIdx.x >> 6);
    if (tile * TILE >= fa.g.d) return;
    const PairDesc pd = fa.g.pairs[blockIdx.y];
    if (tile * TILE + TILE <= fa.g.d) fused_pair_tile<BITS, STALE, INPLACE, NOISE, true>(fa, pd, tile, lane);
    else fused_pair_tile<BITS, STALE, INPLACE, NOISE, false>(fa, pd, tile, lane);
}

// Both reads of a pair are stale: neither node needs the other's current model, only the code the
// other published earlier, so every node is processed on its own.  Same arithmetic and bytes as
// the pair form, but a workgroup touches half as many memory streams at a time (3 float reads, one
// float write, two code streams), and HBM bandwidth on this part falls with the number of
// concurrent streams.
template <int BITS, bool INPLACE, bool NOISE, bool FULL>
__device__ __forceinline__ void fused_node_tile(const FusedArgs &fa, uint32_t node, uint32_t partner, uint32_t age,
                                                uint32_t H, uint64_t tile, uint32_t lane) {
    const GossipArgs &a = fa.g;
    const uint64_t kA = tile * TILE + 4ull * lane, kB = kA + TILE / 2;
    const bool inA = FULL || kA < a.d, inB = FULL || kB < a.d;
    const uint64_t lA = inA ? kA : a.d - 4, lB = inB ? kB : a.d - 4;
    const uint64_t on = (uint64_t)node * a.d;
    float *x = a.X + on;
    const f4 xA = ldg_nt(x + lA), xB = ldg_nt(x + lB);
    const f4 aA = ldg_nt(fa.A + on + lA), aB = ldg_nt(fa.A + on + lB);
    const f4 cA = ldg_nt(fa.C + on + lA), cB = ldg_nt(fa.C + on + lB);
    const uint64_t slot_bytes = (uint64_t)a.n * a.row_bytes;
    const uint8_t *src = a.ring + ((a.slot_now + a.ring_depth - age) % a.ring_depth) * slot_bytes + partner * a.row_bytes;
    const uint64_t seenA = load_code<BITS>(src, lA / 4), seenB = load_code<BITS>(src, lB / 4);
    f4 wA = xA, wB = xB;
    diag_steps<NOISE>(wA, wB, aA, aB, cA, cB, node, tile, lane, H, fa.lr, fa.sigma, a.seed, a.event);
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const f4 qA = INPLACE ? wA : xA, qB = INPLACE ? wB : xB;
    const f4 dA = INPLACE ? zero : wA - xA, dB = INPLACE ? zero : wB - xB;
    const LaneRandom r = row_random(a.seed, node, a.event, tile, lane);
    bool clampedA = false, clampedB = false;
    int fails = 0;
    int zA[4], zB[4];
    const ReadScale rs = read_scale(a, age, a.eps, a.inv_eps);
    const uint64_t codeA = round_float4<BITS>(qA, r.a0, r.a1, rs.inv_now, zA, clampedA);
    const uint64_t codeB = round_float4<BITS>(qB, r.b0, r.b1, rs.inv_now, zB, clampedB);
    f4 oA, oB;
    if (a.eps_slots) {
        float far = 0.f;
        oA = averaged_mixed<BITS>(zA, seenA, qA, dA, rs.eps_now, rs.eps_old, rs.inv_old, nullptr, fails, clampedA, far, inA);
        oB = averaged_mixed<BITS>(zB, seenB, qB, dB, rs.eps_now, rs.eps_old, rs.inv_old, nullptr, fails, clampedB, far, inB);
        report_far(a.far_bits, far);
    } else {
        const float half_eps = 0.5f * rs.eps_now;
        oA = averaged<BITS>(zA, seenA, qA, dA, rs.inv_now, half_eps, nullptr, fails, clampedA);
        oB = averaged<BITS>(zB, seenB, qB, dB, rs.inv_now, half_eps, nullptr, fails, clampedB);
    }
    uint8_t *pub = a.ring + a.slot_now * slot_bytes + node * a.row_bytes;
    if (inA) { stg_nt(x + kA, oA); store_code<BITS>(pub, kA / 4, codeA); }
    if (inB) { stg_nt(x + kB, oB); store_code<BITS>(pub, kB / 4, codeB); }
    report(a.counters, 0, (inA && clampedA) || (inB && clampedB));
}

template <int BITS, bool INPLACE, bool NOISE>
__global__ __launch_bounds__(FWAVES * 64) void fused_nodes_kernel(const FusedArgs fa) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = (uint64_t)blockIdx.x * FWAVES + (threadIdx.x >> 6);
    if (tile * TILE >= fa.g.d) return;
    const PairDesc pd = fa.g.pairs[blockIdx.y >> 1];              // two rows of the grid per pair
    const bool second = blockIdx.y & 1u;
    const uint32_t node = second ? pd.nj : pd.ni, partner = second ? pd.ni : pd.nj;
    const uint32_t age = (pd.flags >> (second ? 8 : 0)) & 0xFFu, H = (pd.steps >> (second ? 8 : 0)) & 0xFFu;
    if (tile * TILE + TILE <= fa.g.d) fused_node_tile<BITS, INPLACE, NOISE, true>(fa, node, partner, age, H, tile, lane);
    else fused_node_tile<BITS, INPLACE, NOISE, false>(fa, node, partner, age, H, tile, lane);
}

// Unmatched nodes: take the local steps and adopt the result; publish the code of the model
// that a partner would have read (the pre-step model when the apply is deferred).
template <int BITS, bool INPLACE, bool NOISE>
__global__ __launch_bounds__(FWAVES * 64) void fused_singles_kernel(const FusedArgs fa) {
    const GossipArgs &a = fa.g;
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = (uint64_t)blockIdx.x * FWAVES + (threadIdx.x >> 6);
    if (tile * TILE >= a.d) return;
    const uint64_t kA = tile * TILE + 4ull * lane, kB = kA + TILE / 2;
    const bool inA = kA < a.d, inB = kB < a.d;
    const uint64_t lA = inA ? kA : a.d - 4, lB = inB ? kB : a.d - 4;
    const uint32_t entry = a.singles[blockIdx.y];
    const uint32_t u = entry & SINGLE_NODE_MASK, Hu = (entry >> 16) & 0xFFu;
    const uint64_t ou = (uint64_t)u * a.d;
    float *xu = a.X + ou;
    const f4 xA = ldg_nt(xu + lA), xB = ldg_nt(xu + lB);
    f4 wA = xA, wB = xB;
    diag_steps<NOISE>(wA, wB, ldg_nt(fa.A + ou + lA), ldg_nt(fa.A + ou + lB), ldg_nt(fa.C + ou + lA), ldg_nt(fa.C + ou + lB), u, tile,
                      lane, Hu, fa.lr, fa.sigma, a.seed, a.event);
    if constexpr (BITS > 0) {
        const LaneRandom r = row_random(a.seed, u, a.event, tile, lane);
        bool clampedA = false, clampedB = false;
        int z[4];
        const float inv_now = read_scale(a, 0, a.eps, a.inv_eps).inv_now;
        const uint64_t cA = round_float4<BITS>(INPLACE ? wA : xA, r.a0, r.a1, inv_now, z, clampedA);
        const uint64_t cB = round_float4<BITS>(INPLACE ? wB : xB, r.b0, r.b1, inv_now, z, clampedB);
        uint8_t *pub = a.ring + a.slot_now * ((uint64_t)a.n * a.row_bytes) + u * a.row_bytes;
        if (inA) store_code<BITS>(pub, kA / 4, cA);
        if (inB) store_code<BITS>(pub, kB / 4, cB);
        report(a.counters, 0, (inA && clampedA) || (inB && clampedB));
    }
    if (inA) stg_nt(xu + kA, wA);
    if (inB) stg_nt(xu + kB, wB);
}

template <int BITS, bool INPLACE, bool NOISE>
static void launch_pairs_stale(const FusedArgs &fa, int stale_mode, dim3 grid, hipStream_t st) {
    switch (stale_mode) {
        case 0: fused_pairs_kernel<BITS, 0, INPLACE, NOISE><<<grid, FWAVES * 64, 0, st>>>(fa); break;
        case 1:   // both reads stale: one grid row per node
            fused_nodes_kernel<BITS, INPLACE, NOISE><<<dim3(grid.x, 2 * grid.y, 1), FWAVES * 64, 0, st>>>(fa);
            break;
        case 3: fused_pairs_kernel<BITS, 3, INPLACE, NOISE><<<grid, FWAVES * 64, 0, st>>>(fa); break;
        default: fused_pairs_kernel<BITS, 2, INPLACE, NOISE><<<grid, FWAVES * 64, 0, st>>>(fa); break;
    }
}

template <int BITS>
static void launch_bits(const FusedArgs &fa, bool inplace, bool noise, int stale_mode, uint32_t npairs,
                        uint32_t nsingles, bool singles, hipStream_t st) {
    const uint64_t tiles = (fa.g.d + TILE - 1) / TILE;
    const unsigned gx = (unsigned)((tiles + FWAVES - 1) / FWAVES);
    if (!singles) {
        const dim3 grid(gx, npairs, 1);
        if (inplace) { if (noise) launch_pairs_stale<BITS, true, true>(fa, stale_mode, grid, st); else launch_pairs_stale<BITS, true, false>(fa, stale_mode, grid, st); }
        else { if (noise) launch_pairs_stale<BITS, false, true>(fa, stale_mode, grid, st); else launch_pairs_stale<BITS, false, false>(fa, stale_mode, grid, st); }
    } else {
        const dim3 grid(gx, nsingles, 1);
        if (inplace) { if (noise) fused_singles_kernel<BITS, true, true><<<grid, FWAVES * 64, 0, st>>>(fa); else fused_singles_kernel<BITS, true, false><<<grid, FWAVES * 64, 0, st>>>(fa); }
        else { if (noise) fused_singles_kernel<BITS, false, true><<<grid, FWAVES * 64, 0, st>>>(fa); else fused_singles_kernel<BITS, false, false><<<grid, FWAVES * 64, 0, st>>>(fa); }
    }
}

static hipError_t dispatch(const GossipArgs &g, const DiagObjective &o, uint32_t bits, bool inplace, uint32_t H,
                           float lr, int stale_mode, uint32_t npairs, uint32_t nsingles, bool singles, hipStream_t st) {
    (void)H;
    FusedArgs fa{g, o.a, o.c, o.sigma, lr};
    const bool noise = o.sigma != 0.f;
    switch (bits) {
        case 2: launch_bits<2>(fa, inplace, noise, stale_mode, npairs, nsingles, singles, st); break;
        case 4: launch_bits<4>(fa, inplace, noise, stale_mode, npairs, nsingles, singles, st); break;
        case 8: launch_bits<8>(fa, inplace, noise, stale_mode, npairs, nsingles, singles, st); break;
        case 16: launch_bits<16>(fa, inplace, noise, stale_mode, npairs, nsingles, singles, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_fused_pairs(const GossipArgs &g, const DiagObjective &o, uint32_t bits, bool inplace, uint32_t H,
                              float lr, int stale_mode, uint32_t npairs, hipStream_t st) {
    if (npairs == 0) return hipSuccess;
    return dispatch(g, o, bits, inplace, H, lr, stale_mode, npairs, 0, false, st);
}

hipError_t launch_fused_singles(const GossipArgs &g, const DiagObjective &o, uint32_t bits, bool inplace, uint32_t H,
                                float lr, uint32_t nsingles, hipStream_t st) {
    if (nsingles == 0) return hipSuccess;
    return dispatch(g, o, bits, inplace, H, lr, 0, 0, nsingles, true, st);
}

}  // namespace swarm
