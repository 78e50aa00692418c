// One wave's tile of a gossip round (Section 3, "Parallel Execution"; Algorithm 1, the decode /
// average / write-back lines), shared by every round kernel: the gossip pass that reads the pending
// local steps from the live copies W, and the one-pass round that takes the H local steps of a
// per-coordinate objective in registers.  For each matched node, one pass over its row does
// stochastic rounding to the lattice, b-bit code packing and publication, decoding of the partner's
// (possibly stale) code against the reader's own model, averaging, and adding the pending update:
//   deferred apply:  z = SR(X),  X' = eps (z_i + z_j')/2 + (w - X)      (the paper's rule)
//   in-place apply:  z = SR(w),  X' = eps (z_i + z_j')/2, decoded against w   (one-pass round only)
//
// Thread layout (wave64): one wave owns a tile of 512 consecutive coordinates = 128 float4; lane l
// holds float4 number l and l+64 of the tile, so every 128-bit load and store of a wave covers 1 KiB
// of consecutive addresses.  One Philox call serves the 8 coordinates [8g, 8g+8) = float4 2g and
// 2g+1; the even lane of each lane pair generates the call for group l/2, the odd lane the call for
// group 32 + l/2, and the two swap halves through a DPP quad permute.
// The tile index is a scalar (the wave number is read from the first lane), so row bases live in
// scalar registers and a lane contributes only its 16-byte offset to every address.
#pragma once
#include "diag_steps.hpp"
#include "gossip_common.hpp"
#include "objectives.h"

namespace swarm {

struct RoundArgs {
    GossipArgs g;
    const float *A, *C;       // n x d objective data (one-pass round only)
    float sigma, lr;
};

// Where a node's pending update comes from.
enum : int {
    SRC_NONE = 0,         // nothing pending
    SRC_LIVE = 1,         // W - X for every node of the launch
    SRC_FLAGGED = 2,      // W - X where the descriptor flags the node
    SRC_STEPS_NOISY = 3,  // H local steps of the diagonal objective in registers, with gradient noise
    SRC_STEPS = 4         // the same without noise
};
__host__ __device__ constexpr bool steps_inside(int src) { return src >= SRC_STEPS_NOISY; }

// Tile of this wave: scalar tile index, lane, and the lane's two float4 positions in the row.
// FULL: the tile lies wholly inside the row, so no lane needs a guard and every load is issued before
// the first use; the ragged last tile of a row takes the guarded variant, where lanes past the end of
// the row load the row's last float4 instead (never stored).
struct TilePos {
    uint64_t tile;        // uniform
    uint64_t base;        // first coordinate of the tile (uniform)
    uint32_t lane;
    uint32_t cA, cB;      // the lane's two float4 as coordinate offsets inside the tile (where they are stored)
    uint32_t oA, oB;      // where they are loaded from
    bool inA, inB;
};
template <bool FULL>
__device__ __forceinline__ TilePos tile_pos(uint64_t tile, uint32_t lane, uint64_t d) {
    TilePos t;
    t.tile = tile; t.lane = lane;
    t.base = tile * TILE;
    t.cA = 4u * lane;
    t.cB = t.cA + TILE / 2;
    t.inA = FULL || t.base + t.cA < d;
    t.inB = FULL || t.base + t.cB < d;
    const uint32_t last = FULL ? 0u : (uint32_t)(d - 4 - t.base);     // the row's last float4 (ragged tile only)
    t.oA = t.inA ? t.cA : last;
    t.oB = t.inB ? t.cB : last;
    return t;
}

// What is read of one node before any arithmetic: its model, and the live copy (u) or the
// objective data a (u) and c (v).
struct NodeRows {
    f4 xA, xB, uA, uB, vA, vB;
};
template <int SRC>
__device__ __forceinline__ NodeRows load_rows(const RoundArgs &ra, uint32_t node, bool pending, const TilePos &t) {
    const GossipArgs &a = ra.g;
    const uint64_t at = (uint64_t)node * a.d + t.base;             // uniform: the lanes add 32-bit offsets
    NodeRows r;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const float *x = a.X + at;
    r.xA = ldg_nt(x, t.oA); r.xB = ldg_nt(x, t.oB);
    r.uA = r.uB = r.vA = r.vB = zero;
    if (steps_inside(SRC)) {
        const float *pa = ra.A + at, *pc = ra.C + at;
        r.uA = ldg_nt(pa, t.oA); r.uB = ldg_nt(pa, t.oB);
        r.vA = ldg_nt(pc, t.oA); r.vB = ldg_nt(pc, t.oB);
    } else if (SRC == SRC_LIVE || (SRC == SRC_FLAGGED && pending)) {
        const float *w = a.W + at;
        r.uA = ldg_nt(w, t.oA); r.uB = ldg_nt(w, t.oB);
    }
    return r;
}

// What the node brings to the exchange: q is rounded to the lattice and serves as decoding key, d is
// added on top of the average.
struct NodeTerms {
    f4 qA, qB, dA, dB;
    f4 wA, wB;            // the model with the node's own steps applied (what an unmatched node adopts)
};
template <int SRC, bool INPLACE>
__device__ __forceinline__ NodeTerms node_terms(const RoundArgs &ra, const NodeRows &r, uint32_t node, bool pending,
                                                uint32_t H, const TilePos &t) {
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    NodeTerms o;
    if (steps_inside(SRC)) {
        f4 wA = r.xA, wB = r.xB;
        diag_steps<SRC == SRC_STEPS_NOISY>(wA, wB, r.uA, r.uB, r.vA, r.vB, node, t.tile, t.lane, H, ra.lr, ra.sigma, ra.g.seed,
                                           ra.g.event);
        o.qA = INPLACE ? wA : r.xA; o.qB = INPLACE ? wB : r.xB;
        o.dA = INPLACE ? zero : wA - r.xA; o.dB = INPLACE ? zero : wB - r.xB;
        o.wA = wA; o.wB = wB;
    } else {
        const bool delta = SRC == SRC_LIVE || (SRC == SRC_FLAGGED && pending);
        o.qA = r.xA; o.qB = r.xB;
        o.dA = delta ? r.uA - r.xA : zero; o.dB = delta ? r.uB - r.xB : zero;
        o.wA = delta ? r.uA : r.xA; o.wB = delta ? r.uB : r.xB;
    }
    return o;
}

// Register row of `node` in ring slot `slot`, at the tile's first code (uniform).
template <int BITS>
__device__ __forceinline__ uint8_t *ring_tile(const GossipArgs &a, uint32_t slot, uint32_t node, const TilePos &t) {
    return a.ring + ((uint64_t)slot * a.n + node) * a.row_bytes + t.base * BITS / 8;
}
__device__ __forceinline__ uint32_t slot_of_age(const GossipArgs &a, uint32_t age) {
    return (a.slot_now + a.ring_depth - age) % a.ring_depth;
}

// Both nodes of a pair in one workgroup row.  STALE: 0 = both reads fresh, 1 = both stale, 2 = per-pair
// flags, 3 = only i's read is stale.
template <int BITS, int SRC, int STALE, bool INPLACE, bool FULL>
__device__ __forceinline__ void round_pair_tile(const RoundArgs &ra, const PairDesc pd, uint64_t tile, uint32_t lane,
                                                float eps, float inv_eps) {
    const GossipArgs &a = ra.g;
    const TilePos t = tile_pos<FULL>(tile, lane, a.d);
    const uint32_t ni = pd.ni, nj = pd.nj;
    const bool pend_i = pd.flags & (1u << 16), pend_j = pd.flags & (1u << 17);
    const uint32_t si = STALE == 0 ? 0u : (pd.flags & 0xFFu);          // age of the code i reads from j
    const uint32_t sj = STALE == 0 ? 0u : ((pd.flags >> 8) & 0xFFu);
    const bool stale_i = STALE == 1 || STALE == 3 || (STALE == 2 && si != 0);
    const bool stale_j = STALE == 1 || (STALE == 2 && sj != 0);

    const NodeRows ri = load_rows<SRC>(ra, ni, pend_i, t), rj = load_rows<SRC>(ra, nj, pend_j, t);
    uint64_t seenjA = 0, seenjB = 0, seeniA = 0, seeniB = 0;       // partner codes as read
    if (stale_i) {   // i reads what j published si rounds ago
        const uint8_t *src = ring_tile<BITS>(a, slot_of_age(a, si), nj, t);
        seenjA = load_tile_code<BITS>(src, t.oA / 4);
        seenjB = load_tile_code<BITS>(src, t.oB / 4);
    }
    if (stale_j) {
        const uint8_t *src = ring_tile<BITS>(a, slot_of_age(a, sj), ni, t);
        seeniA = load_tile_code<BITS>(src, t.oA / 4);
        seeniB = load_tile_code<BITS>(src, t.oB / 4);
    }
    const NodeTerms ti = node_terms<SRC, INPLACE>(ra, ri, ni, pend_i, pd.steps & 0xFFu, t);
    const NodeTerms tj = node_terms<SRC, INPLACE>(ra, rj, nj, pend_j, (pd.steps >> 8) & 0xFFu, t);

    const LaneRandom rndi = row_random(a.seed, ni, a.event, tile, lane);
    const LaneRandom rndj = row_random(a.seed, nj, a.event, tile, lane);
    const ReadScale rsi = read_scale(a, si, eps, inv_eps), rsj = read_scale(a, sj, eps, inv_eps);
    const float inv_now = rsi.inv_now;

    bool clampedA = false, clampedB = false;     // counted per half: lanes past the row end hold a duplicate
    int failsA = 0, failsB = 0;
    int ziA[4], ziB[4], zjA[4], zjB[4];
    const uint64_t ciA = round_float4<BITS>(ti.qA, rndi.a0, rndi.a1, inv_now, ziA, clampedA);
    const uint64_t ciB = round_float4<BITS>(ti.qB, rndi.b0, rndi.b1, inv_now, ziB, clampedB);
    const uint64_t cjA = round_float4<BITS>(tj.qA, rndj.a0, rndj.a1, inv_now, zjA, clampedA);
    const uint64_t cjB = round_float4<BITS>(tj.qB, rndj.b0, rndj.b1, inv_now, zjB, clampedB);
    f4 oiA, oiB, ojA, ojB;
    if (a.eps_slots) {                           // one scale per round: the partner's code may be on an older lattice
        float far = 0.f;
        oiA = averaged_mixed<BITS>(ziA, stale_i ? seenjA : cjA, ti.qA, ti.dA, rsi.eps_now, rsi.eps_old, rsi.inv_old,
                                   stale_i ? nullptr : zjA, failsA, clampedA, far, t.inA);
        oiB = averaged_mixed<BITS>(ziB, stale_i ? seenjB : cjB, ti.qB, ti.dB, rsi.eps_now, rsi.eps_old, rsi.inv_old,
                                   stale_i ? nullptr : zjB, failsB, clampedB, far, t.inB);
        ojA = averaged_mixed<BITS>(zjA, stale_j ? seeniA : ciA, tj.qA, tj.dA, rsj.eps_now, rsj.eps_old, rsj.inv_old,
                                   stale_j ? nullptr : ziA, failsA, clampedA, far, t.inA);
        ojB = averaged_mixed<BITS>(zjB, stale_j ? seeniB : ciB, tj.qB, tj.dB, rsj.eps_now, rsj.eps_old, rsj.inv_old,
                                   stale_j ? nullptr : ziB, failsB, clampedB, far, t.inB);
        report_far(a.far_bits, far);
    } else {
        const float half_eps = 0.5f * rsi.eps_now;
        oiA = averaged<BITS>(ziA, stale_i ? seenjA : cjA, ti.qA, ti.dA, inv_now, half_eps, stale_i ? nullptr : zjA, failsA, clampedA);
        oiB = averaged<BITS>(ziB, stale_i ? seenjB : cjB, ti.qB, ti.dB, inv_now, half_eps, stale_i ? nullptr : zjB, failsB, clampedB);
        ojA = averaged<BITS>(zjA, stale_j ? seeniA : ciA, tj.qA, tj.dA, inv_now, half_eps, stale_j ? nullptr : ziA, failsA, clampedA);
        ojB = averaged<BITS>(zjB, stale_j ? seeniB : ciB, tj.qB, tj.dB, inv_now, half_eps, stale_j ? nullptr : ziB, failsB, clampedB);
    }
    float *xi = a.X + (uint64_t)ni * a.d + t.base, *xj = a.X + (uint64_t)nj * a.d + t.base;
    uint8_t *pub_i = ring_tile<BITS>(a, a.slot_now, ni, t), *pub_j = ring_tile<BITS>(a, a.slot_now, nj, t);
    if (t.inA) {
        stg_nt(xi, t.cA, oiA); stg_nt(xj, t.cA, ojA);
        store_tile_code<BITS>(pub_i, t.cA / 4, ciA); store_tile_code<BITS>(pub_j, t.cA / 4, cjA);
    }
    if (t.inB) {
        stg_nt(xi, t.cB, oiB); stg_nt(xj, t.cB, ojB);
        store_tile_code<BITS>(pub_i, t.cB / 4, ciB); store_tile_code<BITS>(pub_j, t.cB / 4, cjB);
    }
    report(a.counters, (t.inA ? failsA : 0) + (t.inB ? failsB : 0), (t.inA && clampedA) || (t.inB && clampedB));
}

// Both reads of a pair are stale: each node only needs its own rows and the code its partner published
// earlier, so it is processed on its own -- half as many concurrent memory streams per workgroup as the
// pair form (HBM bandwidth on this part falls with the number of concurrent streams), same arithmetic
// and bytes.
template <int BITS, int SRC, bool INPLACE, bool FULL>
__device__ __forceinline__ void round_node_tile(const RoundArgs &ra, uint32_t node, uint32_t partner, uint32_t age,
                                                bool pending, uint32_t H, uint64_t tile, uint32_t lane) {
    const GossipArgs &a = ra.g;
    const TilePos t = tile_pos<FULL>(tile, lane, a.d);
    const NodeRows r = load_rows<SRC>(ra, node, pending, t);
    const uint8_t *src = ring_tile<BITS>(a, slot_of_age(a, age), partner, t);
    const uint64_t seenA = load_tile_code<BITS>(src, t.oA / 4), seenB = load_tile_code<BITS>(src, t.oB / 4);
    const NodeTerms m = node_terms<SRC, INPLACE>(ra, r, node, pending, H, t);
    const LaneRandom rnd = row_random(a.seed, node, a.event, tile, lane);
    const ReadScale rs = read_scale(a, age, a.eps, a.inv_eps);
    bool clampedA = false, clampedB = false;
    int fails = 0;
    int zA[4], zB[4];
    const uint64_t codeA = round_float4<BITS>(m.qA, rnd.a0, rnd.a1, rs.inv_now, zA, clampedA);
    const uint64_t codeB = round_float4<BITS>(m.qB, rnd.b0, rnd.b1, rs.inv_now, zB, clampedB);
    f4 oA, oB;
    if (a.eps_slots) {
        float far = 0.f;
        oA = averaged_mixed<BITS>(zA, seenA, m.qA, m.dA, rs.eps_now, rs.eps_old, rs.inv_old, nullptr, fails, clampedA, far, t.inA);
        oB = averaged_mixed<BITS>(zB, seenB, m.qB, m.dB, rs.eps_now, rs.eps_old, rs.inv_old, nullptr, fails, clampedB, far, t.inB);
        report_far(a.far_bits, far);
    } else {
        const float half_eps = 0.5f * rs.eps_now;
        oA = averaged<BITS>(zA, seenA, m.qA, m.dA, rs.inv_now, half_eps, nullptr, fails, clampedA);
        oB = averaged<BITS>(zB, seenB, m.qB, m.dB, rs.inv_now, half_eps, nullptr, fails, clampedB);
    }
    float *x = a.X + (uint64_t)node * a.d + t.base;
    uint8_t *pub = ring_tile<BITS>(a, a.slot_now, node, t);
    if (t.inA) { stg_nt(x, t.cA, oA); store_tile_code<BITS>(pub, t.cA / 4, codeA); }
    if (t.inB) { stg_nt(x, t.cB, oB); store_tile_code<BITS>(pub, t.cB / 4, codeB); }
    report(a.counters, 0, (t.inA && clampedA) || (t.inB && clampedB));
}

// Unmatched node: publish the code of the model a partner would have read (the pre-step model when the
// apply is deferred), then adopt the node's own steps.
template <int BITS, int SRC, bool INPLACE>
__device__ __forceinline__ void round_single_tile(const RoundArgs &ra, uint32_t entry, uint64_t tile, uint32_t lane) {
    const GossipArgs &a = ra.g;
    const TilePos t = tile_pos<false>(tile, lane, a.d);
    const uint32_t u = entry & SINGLE_NODE_MASK;
    const bool pending = entry & SINGLE_PENDING;
    if (BITS == 0 && !steps_inside(SRC) && !pending) return;          // nothing to publish, nothing to adopt
    const NodeRows r = load_rows<SRC>(ra, u, pending, t);
    const NodeTerms m = node_terms<SRC, INPLACE>(ra, r, u, pending, (entry >> 16) & 0xFFu, t);
    if constexpr (BITS > 0) {
        const LaneRandom rnd = row_random(a.seed, u, a.event, tile, lane);
        bool clampedA = false, clampedB = false;
        int z[4];
        const float inv_now = read_scale(a, 0, a.eps, a.inv_eps).inv_now;
        const uint64_t cA = round_float4<BITS>(m.qA, rnd.a0, rnd.a1, inv_now, z, clampedA);
        const uint64_t cB = round_float4<BITS>(m.qB, rnd.b0, rnd.b1, inv_now, z, clampedB);
        uint8_t *pub = ring_tile<BITS>(a, a.slot_now, u, t);
        if (t.inA) store_tile_code<BITS>(pub, t.cA / 4, cA);
        if (t.inB) store_tile_code<BITS>(pub, t.cB / 4, cB);
        report(a.counters, 0, (t.inA && clampedA) || (t.inB && clampedB));
    }
    if (steps_inside(SRC) || pending) {          // X_u <- w_u: the live copy itself, or the steps just taken
        float *xu = a.X + (uint64_t)u * a.d + t.base;
        if (t.inA) stg_nt(xu, t.cA, m.wA);
        if (t.inB) stg_nt(xu, t.cB, m.wB);
    }
}

// Kernel bodies (the __global__ wrappers keep their own names in gossip.hip and fused.hip).
template <int BITS, int SRC, int STALE, bool INPLACE>
__device__ __forceinline__ void round_pairs_body(const RoundArgs &ra) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = wave_tile(WAVES);
    if (tile * TILE >= ra.g.d) return;
    const PairDesc pd = pair_desc(ra.g, blockIdx.y);               // uniform: one scalar load
    float eps = ra.g.eps, inv_eps = ra.g.inv_eps;
    if (ra.g.pair_linf) {                                          // the pair's own scale from its distance
        const uint32_t *stripes = ra.g.pair_linf + blockIdx.y * PAIR_STRIPES;      // uniform: scalar loads
        uint32_t bits = 0u;
#pragma unroll
        for (uint32_t k = 0; k < PAIR_STRIPES; ++k) bits = max(bits, stripes[k]);
        eps = pair_scale(__uint_as_float(bits), BITS);
        inv_eps = 1.0f / eps;
    }
    if (tile * TILE + TILE <= ra.g.d) round_pair_tile<BITS, SRC, STALE, INPLACE, true>(ra, pd, tile, lane, eps, inv_eps);
    else round_pair_tile<BITS, SRC, STALE, INPLACE, false>(ra, pd, tile, lane, eps, inv_eps);
}

template <int BITS, int SRC, bool INPLACE>
__device__ __forceinline__ void round_nodes_body(const RoundArgs &ra) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = wave_tile(WAVES);
    if (tile * TILE >= ra.g.d) return;
    const PairDesc pd = pair_desc(ra.g, blockIdx.y >> 1);          // two rows of the grid per pair
    const bool second = blockIdx.y & 1u;
    const uint32_t node = second ? pd.nj : pd.ni, partner = second ? pd.ni : pd.nj;
    const uint32_t age = (pd.flags >> (second ? 8 : 0)) & 0xFFu, H = (pd.steps >> (second ? 8 : 0)) & 0xFFu;
    const bool pending = pd.flags & (second ? 1u << 17 : 1u << 16);
    if (tile * TILE + TILE <= ra.g.d) round_node_tile<BITS, SRC, INPLACE, true>(ra, node, partner, age, pending, H, tile, lane);
    else round_node_tile<BITS, SRC, INPLACE, false>(ra, node, partner, age, pending, H, tile, lane);
}

template <int BITS, int SRC, bool INPLACE>
__device__ __forceinline__ void round_singles_body(const RoundArgs &ra) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = wave_tile(WAVES);
    if (tile * TILE >= ra.g.d) return;
    round_single_tile<BITS, SRC, INPLACE>(ra, single_desc(ra.g, blockIdx.y), tile, lane);
}

inline dim3 tile_grid(uint64_t d, uint32_t rows) {
    const uint64_t tiles = (d + TILE - 1) / TILE;
    return dim3((unsigned)((tiles + WAVES - 1) / WAVES), rows, 1);
}

}  // namespace swarm
