// Multi-resolution registers (proof of Corollary 2.1, second case, and its item 3): a node that
// does not know who will read its code, or how far that reader's key is, writes the code for every
// resolution into its own register, and a reader fetches only the prefix it needs.  Here the codes
// are nested -- the b low bits of a 16-bit residue are the b-bit code -- so a register row holds
//   plane 0: bits 0-3 of every coordinate (d/2 bytes),  plane 1: bits 4-7 (d/2 bytes),
//   plane 2: bits 8-15 (d bytes),  then one 64-bit checksum per tile of 512 coordinates,
// and a reader fetches planes until the decoded tile has the writer's checksum (the confirmation the
// interactive protocol gets from the receiver's reply).  The checksum is two 32-bit sums of
// z * weight with pseudo-random odd weights per position: a failed decode is off by +2^b in some
// coordinates and -2^b in others, which weights linear in the position would cancel too often.  A wave owns exactly one checksum tile, so
// the loop over levels is wave-uniform: plane 0 is the only code traffic unless a tile escalates.
// The kernels are the round kernels of gossip.hip / fused.hip with this register format:
// LOCAL = the H local steps of a diagonal-quadratic objective are taken in registers (one-pass
// round); otherwise the live copy W is read where a node has pending steps.
#include "diag_steps.hpp"
#include "gossip_common.hpp"
#include "objectives.h"

namespace swarm {

struct PrefixArgs {
    GossipArgs g;
    const float *A, *C;       // n x d objective data (LOCAL only)
    float sigma, lr;
};

// Register row of `node` in ring slot `slot`.
struct Register {
    uint8_t *p0, *p1, *p2;
    uint2 *checks;
};
__device__ __forceinline__ Register register_of(const GossipArgs &a, uint32_t slot, uint32_t node) {
    uint8_t *base = a.ring + ((uint64_t)slot * a.n + node) * a.row_bytes;
    return Register{base, base + a.d / 2, base + a.d, (uint2 *)(base + 2 * a.d)};
}

// Sum over the wave as a scalar: four cross-lane adds inside each row of 16 lanes (data-parallel
// primitives, no LDS round trip), then the four row sums through lane reads.
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    v += (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    v += (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x141, 0xF, 0xF, true);   // row_half_mirror
    v += (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x140, 0xF, 0xF, true);   // row_mirror
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) + (uint32_t)__builtin_amdgcn_readlane((int)v, 16) +
           (uint32_t)__builtin_amdgcn_readlane((int)v, 32) + (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}

// The two odd weights of coordinate j of a tile: x = (2j+1) 0x9E3779B1; x ^= x >> 15; x *= 0x85EBCA6B;
// x ^= x >> 13; w1 = x | 1; y = x 0xC2B2AE35; y ^= y >> 16; w2 = y | 1.  Tabulated at compile time
// (4 KiB, read-only, stays in cache): hashing eight positions per lane in every wave cost more
// vector ALU time than the rest of the checksum.
struct WeightTable {
    uint32_t w[PREFIX_TILE][2];
    constexpr WeightTable() : w{} {
        for (uint32_t j = 0; j < PREFIX_TILE; ++j) {
            uint32_t x = (2u * j + 1u) * 0x9E3779B1u;
            x ^= x >> 15;
            x *= 0x85EBCA6Bu;
            x ^= x >> 13;
            uint32_t y = x * 0xC2B2AE35u;
            y ^= y >> 16;
            w[j][0] = x | 1u;
            w[j][1] = y | 1u;
        }
    }
};
__device__ const WeightTable WEIGHTS{};

// Weights of the lane's eight positions (float4 number lane and lane + 64 of the tile).
struct LaneWeights { uint2 a[4], b[4]; };
__device__ __forceinline__ LaneWeights lane_weights(uint32_t lane) {
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    const u4 *ta = (const u4 *)&WEIGHTS.w[4u * lane][0], *tb = (const u4 *)&WEIGHTS.w[256u + 4u * lane][0];
    const u4 a0 = ta[0], a1 = ta[1], b0 = tb[0], b1 = tb[1];
    LaneWeights w;
    w.a[0] = uint2{a0.x, a0.y}; w.a[1] = uint2{a0.z, a0.w}; w.a[2] = uint2{a1.x, a1.y}; w.a[3] = uint2{a1.z, a1.w};
    w.b[0] = uint2{b0.x, b0.y}; w.b[1] = uint2{b0.z, b0.w}; w.b[2] = uint2{b1.x, b1.y}; w.b[3] = uint2{b1.z, b1.w};
    return w;
}

// Both sums over the lane's in-range coordinates of z * weight (mod 2^32), reduced over the wave.
__device__ __forceinline__ uint2 tile_checksum(const int zA[4], const int zB[4], const LaneWeights &w, bool inA, bool inB) {
    uint32_t s1 = 0, s2 = 0;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        if (inA) { s1 += (uint32_t)zA[m] * w.a[m].x; s2 += (uint32_t)zA[m] * w.a[m].y; }
        if (inB) { s1 += (uint32_t)zB[m] * w.b[m].x; s2 += (uint32_t)zB[m] * w.b[m].y; }
    }
    return uint2{wave_sum(s1), wave_sum(s2)};
}
__device__ __forceinline__ bool same(uint2 p, uint2 q) { return p.x == q.x && p.y == q.y; }

// What one node brings to the exchange: its row as read (x), what is rounded and serves as decoding
// key (q), the update added on top of the average (delta), its lattice point and tile checksum.
struct NodeTile {
    f4 qA, qB, dA, dB;
    int zA[4], zB[4];
    uint2 check;
    bool clamped;
};

template <bool LOCAL, bool INPLACE, bool NOISE>
__device__ __forceinline__ NodeTile prepare(const PrefixArgs &pa, uint32_t node, uint32_t H, bool pending,
                                            uint64_t tile, uint32_t lane, uint64_t lA, uint64_t lB, bool inA, bool inB,
                                            const LaneWeights &lw) {
    const GossipArgs &a = pa.g;
    const uint64_t on = (uint64_t)node * a.d;
    const f4 xA = ldg_nt(a.X + on + lA), xB = ldg_nt(a.X + on + lB);
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    NodeTile t;
    if (LOCAL) {
        const f4 aA = ldg_nt(pa.A + on + lA), aB = ldg_nt(pa.A + on + lB);
        const f4 cA = ldg_nt(pa.C + on + lA), cB = ldg_nt(pa.C + on + lB);
        f4 wA = xA, wB = xB;
        diag_steps<NOISE>(wA, wB, aA, aB, cA, cB, node, tile, lane, H, pa.lr, pa.sigma, a.seed, a.event);
        t.qA = INPLACE ? wA : xA; t.qB = INPLACE ? wB : xB;
        t.dA = INPLACE ? zero : wA - xA; t.dB = INPLACE ? zero : wB - xB;
    } else {
        t.qA = xA; t.qB = xB;
        t.dA = zero; t.dB = zero;
        if (pending) { t.dA = ldg_nt(a.W + on + lA) - xA; t.dB = ldg_nt(a.W + on + lB) - xB; }
    }
    const LaneRandom r = row_random(a.seed, node, a.event, tile, lane);
    bool clampedA = false, clampedB = false;
    round_float4<16>(t.qA, r.a0, r.a1, a.inv_eps, t.zA, clampedA);
    round_float4<16>(t.qB, r.b0, r.b1, a.inv_eps, t.zB, clampedB);
    t.clamped = (inA && clampedA) || (inB && clampedB);
    t.check = tile_checksum(t.zA, t.zB, lw, inA, inB);
    return t;
}

// Write the lattice point into the node's own register: three planes and the tile's checksum.
__device__ __forceinline__ void publish(const GossipArgs &a, uint32_t node, const NodeTile &t, uint64_t tile,
                                        uint32_t lane, uint64_t kA, uint64_t kB, bool inA, bool inB) {
    const Register reg = register_of(a, a.slot_now, node);
    auto planes = [&](const int z[4], uint64_t k) {
        uint32_t lo = 0, mid = 0, hi = 0;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint32_t c = (uint32_t)z[m];
            lo |= (c & 15u) << (4 * m);
            mid |= ((c >> 4) & 15u) << (4 * m);
            hi |= ((c >> 8) & 255u) << (8 * m);
        }
        __builtin_nontemporal_store((uint16_t)lo, (uint16_t *)(reg.p0 + k / 2));
        __builtin_nontemporal_store((uint16_t)mid, (uint16_t *)(reg.p1 + k / 2));
        __builtin_nontemporal_store(hi, (uint32_t *)(reg.p2 + k));
    };
    if (inA) planes(t.zA, kA);
    if (inB) planes(t.zB, kB);
    if (lane == 0) {
        __builtin_nontemporal_store(t.check.x, &reg.checks[tile].x);
        __builtin_nontemporal_store(t.check.y, &reg.checks[tile].y);
    }
}

// The three residue widths a reader may stop at.
template <int BITS>
__device__ __forceinline__ uint2 decode_tile(const uint32_t cA[4], const uint32_t cB[4], const int kA[4], const int kB[4],
                                             int zpA[4], int zpB[4], const LaneWeights &lw, bool inA, bool inB) {
    constexpr uint32_t MASK = (1u << BITS) - 1u;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        zpA[m] = decode_near<BITS>(cA[m] & MASK, kA[m]);
        zpB[m] = decode_near<BITS>(cB[m] & MASK, kB[m]);
    }
    return tile_checksum(zpA, zpB, lw, inA, inB);
}

// Decode the partner's lattice point against the own key from the shortest confirmed prefix.
// MEMORY: the partner's register row `src` is read plane by plane; otherwise the partner's point is
// in registers (a fresh read inside one pair: same decisions, no code traffic).  Returns the level.
template <bool MEMORY>
__device__ __forceinline__ int read_prefix(const Register &src, const NodeTile &partner, const NodeTile &me, float inv_eps,
                                           uint64_t tile, const LaneWeights &lw, uint64_t lA, uint64_t lB, bool inA, bool inB,
                                           int zpA[4], int zpB[4], bool &clamped, bool &confirmed) {
    int kA[4], kB[4];
    const float qa[4] = {me.qA.x, me.qA.y, me.qA.z, me.qA.w}, qb[4] = {me.qB.x, me.qB.y, me.qB.z, me.qB.w};
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        kA[m] = key_cell(qa[m], inv_eps, clamped);
        kB[m] = key_cell(qb[m], inv_eps, clamped);
    }
    uint2 want = partner.check;
    if (MEMORY) {
        const uint2 c = src.checks[tile];
        want = uint2{__builtin_amdgcn_readfirstlane(c.x), __builtin_amdgcn_readfirstlane(c.y)};
    }
    uint32_t cA[4], cB[4];
    if (MEMORY) {
        const uint32_t a0 = __builtin_nontemporal_load((const uint16_t *)(src.p0 + lA / 2));
        const uint32_t b0 = __builtin_nontemporal_load((const uint16_t *)(src.p0 + lB / 2));
#pragma unroll
        for (int m = 0; m < 4; ++m) { cA[m] = (a0 >> (4 * m)) & 15u; cB[m] = (b0 >> (4 * m)) & 15u; }
    } else {
#pragma unroll
        for (int m = 0; m < 4; ++m) { cA[m] = (uint32_t)partner.zA[m] & 0xFFFFu; cB[m] = (uint32_t)partner.zB[m] & 0xFFFFu; }
    }
    confirmed = true;
    if (same(decode_tile<4>(cA, cB, kA, kB, zpA, zpB, lw, inA, inB), want)) return 0;
    if (MEMORY) {
        const uint32_t a1 = __builtin_nontemporal_load((const uint16_t *)(src.p1 + lA / 2));
        const uint32_t b1 = __builtin_nontemporal_load((const uint16_t *)(src.p1 + lB / 2));
#pragma unroll
        for (int m = 0; m < 4; ++m) { cA[m] |= ((a1 >> (4 * m)) & 15u) << 4; cB[m] |= ((b1 >> (4 * m)) & 15u) << 4; }
    }
    if (same(decode_tile<8>(cA, cB, kA, kB, zpA, zpB, lw, inA, inB), want)) return 1;
    if (MEMORY) {
        const uint32_t a2 = __builtin_nontemporal_load((const uint32_t *)(src.p2 + lA));
        const uint32_t b2 = __builtin_nontemporal_load((const uint32_t *)(src.p2 + lB));
#pragma unroll
        for (int m = 0; m < 4; ++m) { cA[m] |= ((a2 >> (8 * m)) & 255u) << 8; cB[m] |= ((b2 >> (8 * m)) & 255u) << 8; }
    }
    confirmed = same(decode_tile<16>(cA, cB, kA, kB, zpA, zpB, lw, inA, inB), want);
    return 2;
}

// Tiles that needed more than the first plane, and tiles no level confirmed (one lane per wave, into
// the stripe of its workgroup).
__device__ __forceinline__ void report_level(PrefixStats *stats, int level, bool confirmed, uint64_t tile, uint64_t d,
                                             uint32_t lane) {
    if (lane != 0 || (level == 0 && confirmed)) return;
    PrefixStats *c = stats + ((blockIdx.x + 977u * blockIdx.y) & (PREFIX_STRIPES - 1));
    const unsigned long long coords = (tile + 1) * TILE <= d ? TILE : d - tile * TILE;
    if (level > 0) {
        atomicAdd(&c->tiles[level - 1], 1ull);
        atomicAdd(&c->coords[level - 1], coords);
    }
    if (!confirmed) atomicAdd(&c->unconfirmed, 1ull);
}

// X' = eps (z + z') / 2 + delta for the lane's two float4.
__device__ __forceinline__ void finish(const GossipArgs &a, uint32_t node, const NodeTile &t, const int zpA[4], const int zpB[4],
                                       uint64_t kA, uint64_t kB, bool inA, bool inB) {
    const float half_eps = 0.5f * a.eps;
    float *x = a.X + (uint64_t)node * a.d;
    const f4 oA = {fmaf((float)(t.zA[0] + zpA[0]), half_eps, t.dA.x), fmaf((float)(t.zA[1] + zpA[1]), half_eps, t.dA.y),
                   fmaf((float)(t.zA[2] + zpA[2]), half_eps, t.dA.z), fmaf((float)(t.zA[3] + zpA[3]), half_eps, t.dA.w)};
    const f4 oB = {fmaf((float)(t.zB[0] + zpB[0]), half_eps, t.dB.x), fmaf((float)(t.zB[1] + zpB[1]), half_eps, t.dB.y),
                   fmaf((float)(t.zB[2] + zpB[2]), half_eps, t.dB.z), fmaf((float)(t.zB[3] + zpB[3]), half_eps, t.dB.w)};
    if (inA) stg_nt(x + kA, oA);
    if (inB) stg_nt(x + kB, oB);
}

struct TileGeometry {
    uint64_t tile, kA, kB, lA, lB;
    uint32_t lane;
    bool inA, inB;
};
__device__ __forceinline__ bool geometry(uint64_t d, int waves, TileGeometry &g) {
    g.lane = threadIdx.x & 63u;
    g.tile = wave_tile(waves);
    if (g.tile * TILE >= d) return false;
    g.kA = g.tile * TILE + 4ull * g.lane;
    g.kB = g.kA + TILE / 2;
    g.inA = g.kA < d;
    g.inB = g.kB < d;
    g.lA = g.inA ? g.kA : d - 4;              // past the row end: re-read its last float4 (never stored)
    g.lB = g.inB ? g.kB : d - 4;
    return true;
}

// Both reads of the pair are stale: every node is processed on its own grid row (two per pair).
template <bool LOCAL, bool INPLACE, bool NOISE>
__global__ __launch_bounds__(WAVES * 64) void prefix_nodes_kernel(const PrefixArgs pa) {
    const GossipArgs &a = pa.g;
    TileGeometry g;
    if (!geometry(a.d, WAVES, g)) return;
    const PairDesc pd = pair_desc(a, blockIdx.y >> 1);
    const bool second = blockIdx.y & 1u;
    const uint32_t node = second ? pd.nj : pd.ni, partner = second ? pd.ni : pd.nj;
    const uint32_t age = (pd.flags >> (second ? 8 : 0)) & 0xFFu, H = (pd.steps >> (second ? 8 : 0)) & 0xFFu;
    const bool pending = pd.flags & (second ? 1u << 17 : 1u << 16);
    const LaneWeights lw = lane_weights(g.lane);
    const NodeTile me = prepare<LOCAL, INPLACE, NOISE>(pa, node, H, pending, g.tile, g.lane, g.lA, g.lB, g.inA, g.inB, lw);
    const Register src = register_of(a, (a.slot_now + a.ring_depth - age) % a.ring_depth, partner);
    int zpA[4], zpB[4];
    bool clamped = false, confirmed;
    const int level = read_prefix<true>(src, me, me, a.inv_eps, g.tile, lw, g.lA, g.lB, g.inA, g.inB, zpA, zpB,
                                        clamped, confirmed);
    publish(a, node, me, g.tile, g.lane, g.kA, g.kB, g.inA, g.inB);
    finish(a, node, me, zpA, zpB, g.kA, g.kB, g.inA, g.inB);
    report_level(a.prefix_stats, level, confirmed, g.tile, a.d, g.lane);
    report(a.counters, 0, me.clamped || ((g.inA || g.inB) && clamped));
}

// Any mix of fresh and stale reads: both nodes of the pair in one workgroup row.
template <bool LOCAL, bool INPLACE, bool NOISE>
__global__ __launch_bounds__(WAVES * 64) void prefix_pairs_kernel(const PrefixArgs pa) {
    const GossipArgs &a = pa.g;
    TileGeometry g;
    if (!geometry(a.d, WAVES, g)) return;
    const PairDesc pd = pair_desc(a, blockIdx.y);
    const uint32_t si = pd.flags & 0xFFu, sj = (pd.flags >> 8) & 0xFFu;
    const LaneWeights lw = lane_weights(g.lane);
    const NodeTile ti = prepare<LOCAL, INPLACE, NOISE>(pa, pd.ni, pd.steps & 0xFFu, pd.flags & (1u << 16), g.tile, g.lane,
                                                       g.lA, g.lB, g.inA, g.inB, lw);
    const NodeTile tj = prepare<LOCAL, INPLACE, NOISE>(pa, pd.nj, (pd.steps >> 8) & 0xFFu, pd.flags & (1u << 17), g.tile,
                                                       g.lane, g.lA, g.lB, g.inA, g.inB, lw);
    int zjA[4], zjB[4], ziA[4], ziB[4];          // what i decodes of j, what j decodes of i
    bool clamped = false, conf_i, conf_j;
    int level_i, level_j;
    if (si) level_i = read_prefix<true>(register_of(a, (a.slot_now + a.ring_depth - si) % a.ring_depth, pd.nj), tj, ti,
                                        a.inv_eps, g.tile, lw, g.lA, g.lB, g.inA, g.inB, zjA, zjB, clamped, conf_i);
    else level_i = read_prefix<false>(Register{}, tj, ti, a.inv_eps, g.tile, lw, g.lA, g.lB, g.inA, g.inB, zjA, zjB,
                                      clamped, conf_i);
    if (sj) level_j = read_prefix<true>(register_of(a, (a.slot_now + a.ring_depth - sj) % a.ring_depth, pd.ni), ti, tj,
                                        a.inv_eps, g.tile, lw, g.lA, g.lB, g.inA, g.inB, ziA, ziB, clamped, conf_j);
    else level_j = read_prefix<false>(Register{}, ti, tj, a.inv_eps, g.tile, lw, g.lA, g.lB, g.inA, g.inB, ziA, ziB,
                                      clamped, conf_j);
    int fails = 0;                               // fresh reads: coordinates decoded to another point than the sender's
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        if (!si) fails += (g.inA && zjA[m] != tj.zA[m]) + (g.inB && zjB[m] != tj.zB[m]);
        if (!sj) fails += (g.inA && ziA[m] != ti.zA[m]) + (g.inB && ziB[m] != ti.zB[m]);
    }
    publish(a, pd.ni, ti, g.tile, g.lane, g.kA, g.kB, g.inA, g.inB);
    publish(a, pd.nj, tj, g.tile, g.lane, g.kA, g.kB, g.inA, g.inB);
    finish(a, pd.ni, ti, zjA, zjB, g.kA, g.kB, g.inA, g.inB);
    finish(a, pd.nj, tj, ziA, ziB, g.kA, g.kB, g.inA, g.inB);
    report_level(a.prefix_stats, level_i, conf_i, g.tile, a.d, g.lane);
    report_level(a.prefix_stats, level_j, conf_j, g.tile, a.d, g.lane);
    report(a.counters, fails, ti.clamped || tj.clamped || ((g.inA || g.inB) && clamped));
}

// Unmatched nodes: adopt the own steps, publish the register (later stale reads need it).
template <bool LOCAL, bool INPLACE, bool NOISE>
__global__ __launch_bounds__(WAVES * 64) void prefix_singles_kernel(const PrefixArgs pa) {
    const GossipArgs &a = pa.g;
    TileGeometry g;
    if (!geometry(a.d, WAVES, g)) return;
    const uint32_t entry = single_desc(a, blockIdx.y);
    const uint32_t u = entry & SINGLE_NODE_MASK;
    const NodeTile t = prepare<LOCAL, INPLACE, NOISE>(pa, u, (entry >> 16) & 0xFFu, entry & SINGLE_PENDING, g.tile, g.lane,
                                                      g.lA, g.lB, g.inA, g.inB, lane_weights(g.lane));
    publish(a, u, t, g.tile, g.lane, g.kA, g.kB, g.inA, g.inB);
    float *x = a.X + (uint64_t)u * a.d;
    if (LOCAL || (entry & SINGLE_PENDING)) {     // X_u <- X_u + delta (the rounded model q is X_u, or already X_u + delta)
        if (g.inA) stg_nt(x + g.kA, t.qA + t.dA);
        if (g.inB) stg_nt(x + g.kB, t.qB + t.dB);
    }
    report(a.counters, 0, t.clamped);
}

// One step of Algorithm 1: both registers are written, the initiator i reads j's by prefixes (the
// lattice point is in registers: same decisions as a read from memory), X_i' = average + (W_i - Xhat_i),
// X_j' = average, Xhat_i' = X_i'.  The average goes back into j's register with as many bits as the read
// took (the initiator knows its distance to j's key by then), which only the bit count records.
__global__ __launch_bounds__(WAVES * 64) void prefix_interact_kernel(const GossipArgs a, const SeqDesc *descs, const SeqDesc one) {
    TileGeometry g;
    if (!geometry(a.d, WAVES, g)) return;
    const SeqDesc sd = descs ? descs[blockIdx.y] : one;          // one grid row per interaction
    const uint32_t ni = sd.ni, nj = sd.nj;
    const bool has_delta = sd.flags & SEQ_HAS_DELTA;
    const LaneWeights lw = lane_weights(g.lane);
    const uint64_t oi = (uint64_t)ni * a.d, oj = (uint64_t)nj * a.d;
    NodeTile ti, tj;
    ti.qA = ldg_nt(a.X + oi + g.lA); ti.qB = ldg_nt(a.X + oi + g.lB);
    tj.qA = ldg_nt(a.X + oj + g.lA); tj.qB = ldg_nt(a.X + oj + g.lB);
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    ti.dA = ti.dB = tj.dA = tj.dB = zero;
    if (has_delta) {
        ti.dA = ldg_nt(a.W + oi + g.lA) - ldg_nt(a.Xhat + oi + g.lA);
        ti.dB = ldg_nt(a.W + oi + g.lB) - ldg_nt(a.Xhat + oi + g.lB);
    }
    const LaneRandom ri = row_random(a.seed, ni, sd.event, g.tile, g.lane), rj = row_random(a.seed, nj, sd.event, g.tile, g.lane);
    bool cA = false, cB = false;
    round_float4<16>(ti.qA, ri.a0, ri.a1, a.inv_eps, ti.zA, cA);
    round_float4<16>(ti.qB, ri.b0, ri.b1, a.inv_eps, ti.zB, cB);
    round_float4<16>(tj.qA, rj.a0, rj.a1, a.inv_eps, tj.zA, cA);
    round_float4<16>(tj.qB, rj.b0, rj.b1, a.inv_eps, tj.zB, cB);
    ti.check = tile_checksum(ti.zA, ti.zB, lw, g.inA, g.inB);
    tj.check = tile_checksum(tj.zA, tj.zB, lw, g.inA, g.inB);
    int zjA[4], zjB[4];
    bool clamped = false, confirmed;
    const int level = read_prefix<false>(Register{}, tj, ti, a.inv_eps, g.tile, lw, g.lA, g.lB, g.inA, g.inB, zjA, zjB,
                                         clamped, confirmed);
    int fails = 0;
#pragma unroll
    for (int m = 0; m < 4; ++m) fails += (g.inA && zjA[m] != tj.zA[m]) + (g.inB && zjB[m] != tj.zB[m]);
    publish(a, ni, ti, g.tile, g.lane, g.kA, g.kB, g.inA, g.inB);
    publish(a, nj, tj, g.tile, g.lane, g.kA, g.kB, g.inA, g.inB);
    const float half_eps = 0.5f * a.eps;
    f4 avgA, avgB;
    avgA.x = (float)(ti.zA[0] + zjA[0]) * half_eps; avgA.y = (float)(ti.zA[1] + zjA[1]) * half_eps;
    avgA.z = (float)(ti.zA[2] + zjA[2]) * half_eps; avgA.w = (float)(ti.zA[3] + zjA[3]) * half_eps;
    avgB.x = (float)(ti.zB[0] + zjB[0]) * half_eps; avgB.y = (float)(ti.zB[1] + zjB[1]) * half_eps;
    avgB.z = (float)(ti.zB[2] + zjB[2]) * half_eps; avgB.w = (float)(ti.zB[3] + zjB[3]) * half_eps;
    if (g.inA) { const f4 o = avgA + ti.dA; stg_nt(a.X + oi + g.kA, o); stg_nt(a.Xhat + oi + g.kA, o); stg_nt(a.X + oj + g.kA, avgA); }
    if (g.inB) { const f4 o = avgB + ti.dB; stg_nt(a.X + oi + g.kB, o); stg_nt(a.Xhat + oi + g.kB, o); stg_nt(a.X + oj + g.kB, avgB); }
    report_level(a.prefix_stats, level, confirmed, g.tile, a.d, g.lane);
    if (g.lane == 0 && level > 0) {              // the write-back of the average took the same prefix length
        const unsigned long long coords = (g.tile + 1) * TILE <= a.d ? TILE : a.d - g.tile * TILE;
        atomicAdd(&a.prefix_stats[(blockIdx.x + 977u * blockIdx.y) & (PREFIX_STRIPES - 1)].written_back[level - 1], coords);
    }
    report(a.counters, fails, (g.inA && cA) || (g.inB && cB) || ((g.inA || g.inB) && clamped));
}

hipError_t launch_prefix_interact(const GossipArgs &g, const SeqDesc *descs_dev, SeqDesc one, uint32_t count,
                                  hipStream_t st) {
    if (count == 0) return hipSuccess;
    const uint64_t tiles = (g.d + TILE - 1) / TILE;
    prefix_interact_kernel<<<dim3((unsigned)((tiles + WAVES - 1) / WAVES), count, 1), WAVES * 64, 0, st>>>(g, descs_dev, one);
    return hipGetLastError();
}

template <bool LOCAL, bool INPLACE, bool NOISE>
static void launch_kind(const PrefixArgs &pa, int kind, dim3 grid, hipStream_t st) {
    if (kind == 0) prefix_pairs_kernel<LOCAL, INPLACE, NOISE><<<grid, WAVES * 64, 0, st>>>(pa);
    else if (kind == 1) prefix_nodes_kernel<LOCAL, INPLACE, NOISE><<<dim3(grid.x, 2 * grid.y, 1), WAVES * 64, 0, st>>>(pa);
    else prefix_singles_kernel<LOCAL, INPLACE, NOISE><<<grid, WAVES * 64, 0, st>>>(pa);
}

// kind: 0 = pairs with any mix of fresh and stale reads, 1 = pairs whose reads are both stale (node by
// node), 2 = unmatched nodes.  local: the diagonal objective of the one-pass round, or null.
hipError_t launch_prefix(const GossipArgs &g, const DiagObjective *local, bool inplace, float lr, int kind, uint32_t rows,
                         hipStream_t st) {
    if (rows == 0) return hipSuccess;
    const uint64_t tiles = (g.d + TILE - 1) / TILE;
    const dim3 grid((unsigned)((tiles + WAVES - 1) / WAVES), rows, 1);
    PrefixArgs pa{g, local ? local->a : nullptr, local ? local->c : nullptr, local ? local->sigma : 0.f, lr};
    if (!local) launch_kind<false, false, false>(pa, kind, grid, st);
    else if (inplace) {
        if (local->sigma != 0.f) launch_kind<true, true, true>(pa, kind, grid, st);
        else launch_kind<true, true, false>(pa, kind, grid, st);
    } else {
        if (local->sigma != 0.f) launch_kind<true, false, true>(pa, kind, grid, st);
        else launch_kind<true, false, false>(pa, kind, grid, st);
    }
    return hipGetLastError();
}

}  // namespace swarm
