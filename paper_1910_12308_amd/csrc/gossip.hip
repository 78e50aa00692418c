// Fused quantized gossip pass (Section 3, "Parallel Execution"; Algorithm 1, the
// decode / average / write-back lines): for each matched pair, one pass over the two
// model rows does stochastic rounding to the lattice, b-bit code packing and
// publication, decoding of the partner's (possibly stale) code against the reader's
// own model, averaging, and adding the pending local update.
//
// Thread layout (wave64): one wave owns a tile of 512 consecutive coordinates = 128
// float4; lane l holds float4 number l and l+64 of the tile, so every 128-bit load and
// store of a wave covers 1 KiB of consecutive addresses.  One Philox call serves the 8
// coordinates [8g, 8g+8) = float4 2g and 2g+1; the even lane of each lane pair
// generates the call for group l/2, the odd lane the call for group 32 + l/2, and the
// two swap halves through a DPP quad permute.
#include "gossip_common.hpp"

namespace swarm {

// One wave's tile of one pair.  FULL: the tile lies wholly inside the row, so no lane needs a
// guard and every load is issued before the first use; the ragged last tile of a row takes the
// guarded variant.
template <int BITS, int DELTA, int STALE, bool FULL>
__device__ __forceinline__ void gossip_pair_tile(const GossipArgs &a, const PairDesc pd, uint64_t tile, uint32_t lane,
                                                 float eps, float inv_eps) {
    const uint64_t kA = tile * TILE + 4ull * lane, kB = kA + TILE / 2;
    const bool inA = FULL || kA < a.d, inB = FULL || kB < a.d;
    // Lanes past the end of the row load the row's last float4 instead (never stored).
    const uint64_t lA = inA ? kA : a.d - 4, lB = inB ? kB : a.d - 4;
    const uint32_t ni = pd.ni, nj = pd.nj;
    float *xi = a.X + (uint64_t)ni * a.d, *xj = a.X + (uint64_t)nj * a.d;
    const float *wi = a.W + (uint64_t)ni * a.d, *wj = a.W + (uint64_t)nj * a.d;

    const bool di = DELTA == 1 || (DELTA == 2 && (pd.flags & (1u << 16)));
    const bool dj = DELTA == 1 || (DELTA == 2 && (pd.flags & (1u << 17)));
    const uint32_t si = STALE == 0 ? 0u : (pd.flags & 0xFFu);          // age of the code i reads from j
    const uint32_t sj = STALE == 0 ? 0u : ((pd.flags >> 8) & 0xFFu);
    // STALE: 0 = both reads fresh, 1 = both stale, 2 = per-pair flags, 3 = only i's read is stale
    const bool stale_i = STALE == 1 || STALE == 3 || (STALE == 2 && si != 0);
    const bool stale_j = STALE == 1 || (STALE == 2 && sj != 0);

    const f4 xiA = ldg_nt(xi + lA), xjA = ldg_nt(xj + lA), xiB = ldg_nt(xi + lB), xjB = ldg_nt(xj + lB);
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    f4 wiA = zero, wiB = zero, wjA = zero, wjB = zero;
    if (di) { wiA = ldg_nt(wi + lA); wiB = ldg_nt(wi + lB); }
    if (dj) { wjA = ldg_nt(wj + lA); wjB = ldg_nt(wj + lB); }

    const uint64_t slot_bytes = (uint64_t)a.n * a.row_bytes;
    uint8_t *pub_i = a.ring + a.slot_now * slot_bytes + ni * a.row_bytes;
    uint8_t *pub_j = a.ring + a.slot_now * slot_bytes + nj * a.row_bytes;
    uint64_t seenjA = 0, seenjB = 0, seeniA = 0, seeniB = 0;       // partner codes as read
    if (stale_i) {   // i reads what j published si rounds ago
        const uint8_t *src = a.ring + ((a.slot_now + a.ring_depth - si) % a.ring_depth) * slot_bytes + nj * a.row_bytes;
        seenjA = load_code<BITS>(src, lA / 4);
        seenjB = load_code<BITS>(src, lB / 4);
    }
    if (stale_j) {
        const uint8_t *src = a.ring + ((a.slot_now + a.ring_depth - sj) % a.ring_depth) * slot_bytes + ni * a.row_bytes;
        seeniA = load_code<BITS>(src, lA / 4);
        seeniB = load_code<BITS>(src, lB / 4);
    }

    const LaneRandom ri = row_random(a.seed, ni, a.event, tile, lane);
    const LaneRandom rj = row_random(a.seed, nj, a.event, tile, lane);
    const ReadScale rsi = read_scale(a, si, eps, inv_eps), rsj = read_scale(a, sj, eps, inv_eps);
    const float inv_now = rsi.inv_now;

    bool clampedA = false, clampedB = false;     // counted per half: lanes past the row end hold a duplicate
    int failsA = 0, failsB = 0;
    int ziA[4], ziB[4], zjA[4], zjB[4];
    const uint64_t ciA = round_float4<BITS>(xiA, ri.a0, ri.a1, inv_now, ziA, clampedA);
    const uint64_t ciB = round_float4<BITS>(xiB, ri.b0, ri.b1, inv_now, ziB, clampedB);
    const uint64_t cjA = round_float4<BITS>(xjA, rj.a0, rj.a1, inv_now, zjA, clampedA);
    const uint64_t cjB = round_float4<BITS>(xjB, rj.b0, rj.b1, inv_now, zjB, clampedB);
    const f4 diA = di ? wiA - xiA : zero, diB = di ? wiB - xiB : zero;
    const f4 djA = dj ? wjA - xjA : zero, djB = dj ? wjB - xjB : zero;
    f4 oiA, oiB, ojA, ojB;
    if (a.eps_slots) {                           // one scale per round: the partner's code may be on an older lattice
        float far = 0.f;
        oiA = averaged_mixed<BITS>(ziA, stale_i ? seenjA : cjA, xiA, diA, rsi.eps_now, rsi.eps_old, rsi.inv_old,
                                   stale_i ? nullptr : zjA, failsA, clampedA, far, inA);
        oiB = averaged_mixed<BITS>(ziB, stale_i ? seenjB : cjB, xiB, diB, rsi.eps_now, rsi.eps_old, rsi.inv_old,
                                   stale_i ? nullptr : zjB, failsB, clampedB, far, inB);
        ojA = averaged_mixed<BITS>(zjA, stale_j ? seeniA : ciA, xjA, djA, rsj.eps_now, rsj.eps_old, rsj.inv_old,
                                   stale_j ? nullptr : ziA, failsA, clampedA, far, inA);
        ojB = averaged_mixed<BITS>(zjB, stale_j ? seeniB : ciB, xjB, djB, rsj.eps_now, rsj.eps_old, rsj.inv_old,
                                   stale_j ? nullptr : ziB, failsB, clampedB, far, inB);
        report_far(a.far_bits, far);
    } else {
        const float half_eps = 0.5f * rsi.eps_now;
        oiA = averaged<BITS>(ziA, stale_i ? seenjA : cjA, xiA, diA, inv_now, half_eps, stale_i ? nullptr : zjA, failsA, clampedA);
        oiB = averaged<BITS>(ziB, stale_i ? seenjB : cjB, xiB, diB, inv_now, half_eps, stale_i ? nullptr : zjB, failsB, clampedB);
        ojA = averaged<BITS>(zjA, stale_j ? seeniA : ciA, xjA, djA, inv_now, half_eps, stale_j ? nullptr : ziA, failsA, clampedA);
        ojB = averaged<BITS>(zjB, stale_j ? seeniB : ciB, xjB, djB, inv_now, half_eps, stale_j ? nullptr : ziB, failsB, clampedB);
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

// Both reads of a pair are stale: each node only needs its own rows and the code its partner
// published earlier, so it is processed on its own -- half as many concurrent memory streams per
// workgroup as the pair form, same arithmetic and bytes.
template <int BITS, int DELTA, bool FULL>
__device__ __forceinline__ void gossip_node_tile(const GossipArgs &a, uint32_t node, uint32_t partner, uint32_t age,
                                                 bool pending, uint64_t tile, uint32_t lane) {
    const uint64_t kA = tile * TILE + 4ull * lane, kB = kA + TILE / 2;
    const bool inA = FULL || kA < a.d, inB = FULL || kB < a.d;
    const uint64_t lA = inA ? kA : a.d - 4, lB = inB ? kB : a.d - 4;
    float *x = a.X + (uint64_t)node * a.d;
    const float *w = a.W + (uint64_t)node * a.d;
    const bool delta = DELTA == 1 || (DELTA == 2 && pending);
    const f4 xA = ldg_nt(x + lA), xB = ldg_nt(x + lB);
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    f4 wA = zero, wB = zero;
    if (delta) { wA = ldg_nt(w + lA); wB = ldg_nt(w + lB); }
    const uint64_t slot_bytes = (uint64_t)a.n * a.row_bytes;
    const uint8_t *src = a.ring + ((a.slot_now + a.ring_depth - age) % a.ring_depth) * slot_bytes + partner * a.row_bytes;
    const uint64_t seenA = load_code<BITS>(src, lA / 4), seenB = load_code<BITS>(src, lB / 4);
    const LaneRandom r = row_random(a.seed, node, a.event, tile, lane);
    const ReadScale rs = read_scale(a, age, a.eps, a.inv_eps);
    bool clampedA = false, clampedB = false;
    int fails = 0;
    int zA[4], zB[4];
    const uint64_t codeA = round_float4<BITS>(xA, r.a0, r.a1, rs.inv_now, zA, clampedA);
    const uint64_t codeB = round_float4<BITS>(xB, r.b0, r.b1, rs.inv_now, zB, clampedB);
    const f4 dA = delta ? wA - xA : zero, dB = delta ? wB - xB : zero;
    f4 oA, oB;
    if (a.eps_slots) {
        float far = 0.f;
        oA = averaged_mixed<BITS>(zA, seenA, xA, dA, rs.eps_now, rs.eps_old, rs.inv_old, nullptr, fails, clampedA, far, inA);
        oB = averaged_mixed<BITS>(zB, seenB, xB, dB, rs.eps_now, rs.eps_old, rs.inv_old, nullptr, fails, clampedB, far, inB);
        report_far(a.far_bits, far);
    } else {
        const float half_eps = 0.5f * rs.eps_now;
        oA = averaged<BITS>(zA, seenA, xA, dA, rs.inv_now, half_eps, nullptr, fails, clampedA);
        oB = averaged<BITS>(zB, seenB, xB, dB, rs.inv_now, half_eps, nullptr, fails, clampedB);
    }
    uint8_t *pub = a.ring + a.slot_now * slot_bytes + node * a.row_bytes;
    if (inA) { stg_nt(x + kA, oA); store_code<BITS>(pub, kA / 4, codeA); }
    if (inB) { stg_nt(x + kB, oB); store_code<BITS>(pub, kB / 4, codeB); }
    report(a.counters, 0, (inA && clampedA) || (inB && clampedB));
}

template <int BITS, int DELTA>
__global__ __launch_bounds__(WAVES * 64) void gossip_nodes_kernel(const GossipArgs a) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = (uint64_t)blockIdx.x * WAVES + (threadIdx.x >> 6);
    if (tile * TILE >= a.d) return;
    const PairDesc pd = a.pairs[blockIdx.y >> 1];                  // two rows of the grid per pair
    const bool second = blockIdx.y & 1u;
    const uint32_t node = second ? pd.nj : pd.ni, partner = second ? pd.ni : pd.nj;
    const uint32_t age = (pd.flags >> (second ? 8 : 0)) & 0xFFu;
    const bool pending = pd.flags & (second ? 1u << 17 : 1u << 16);
    if (tile * TILE + TILE <= a.d) gossip_node_tile<BITS, DELTA, true>(a, node, partner, age, pending, tile, lane);
    else gossip_node_tile<BITS, DELTA, false>(a, node, partner, age, pending, tile, lane);
}

template <int BITS, int DELTA, int STALE>
__global__ __launch_bounds__(WAVES * 64) void gossip_pairs_kernel(const GossipArgs a) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = (uint64_t)blockIdx.x * WAVES + (threadIdx.x >> 6);
    if (tile * TILE >= a.d) return;
    const PairDesc pd = a.pairs[blockIdx.y];                       // uniform: one scalar load
    float eps = a.eps, inv_eps = a.inv_eps;
    if (a.pair_linf) {                                             // the pair's own scale from its distance
        eps = pair_scale(__uint_as_float(a.pair_linf[blockIdx.y]), BITS);
        inv_eps = 1.0f / eps;
    }
    if (tile * TILE + TILE <= a.d) gossip_pair_tile<BITS, DELTA, STALE, true>(a, pd, tile, lane, eps, inv_eps);
    else gossip_pair_tile<BITS, DELTA, STALE, false>(a, pd, tile, lane, eps, inv_eps);
}

// Q = identity (Corollary 4.2): plain pairwise averaging plus the pending update.
template <int DELTA>
__global__ __launch_bounds__(WAVES * 64) void average_pairs_kernel(const GossipArgs a) {
    const uint64_t k = ((uint64_t)blockIdx.x * (WAVES * 64) + threadIdx.x) * 4;
    if (k >= a.d) return;
    const PairDesc pd = a.pairs[blockIdx.y];
    const uint32_t ni = pd.ni, nj = pd.nj;
    float *xi = a.X + (uint64_t)ni * a.d + k, *xj = a.X + (uint64_t)nj * a.d + k;
    const f4 vi = ldg_nt(xi), vj = ldg_nt(xj);
    f4 di = {0.f, 0.f, 0.f, 0.f}, dj = di;
    if (DELTA == 1 || (DELTA == 2 && (pd.flags & (1u << 16)))) di = ldg_nt(a.W + (uint64_t)ni * a.d + k) - vi;
    if (DELTA == 1 || (DELTA == 2 && (pd.flags & (1u << 17)))) dj = ldg_nt(a.W + (uint64_t)nj * a.d + k) - vj;
    const f4 avg = 0.5f * (vi + vj);
    stg_nt(xi, avg + di);
    stg_nt(xj, avg + dj);
}

// Unmatched nodes: publish the code of X_u, then apply the node's own pending steps.
template <int BITS>
__global__ __launch_bounds__(WAVES * 64) void gossip_singles_kernel(const GossipArgs a) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = (uint64_t)blockIdx.x * WAVES + (threadIdx.x >> 6);
    const uint64_t kA = tile * TILE + 4ull * lane, kB = kA + TILE / 2;
    const bool inA = kA < a.d, inB = kB < a.d;
    if (tile * TILE >= a.d) return;
    const uint32_t entry = a.singles[blockIdx.y];
    const uint32_t u = entry & SINGLE_NODE_MASK;
    float *xu = a.X + (uint64_t)u * a.d;
    const float *wu = a.W + (uint64_t)u * a.d;
    const bool pend = entry & SINGLE_PENDING;
    if constexpr (BITS > 0) {
        const f4 zero = {0.f, 0.f, 0.f, 0.f};
        const f4 xA = inA ? ldg_nt(xu + kA) : zero, xB = inB ? ldg_nt(xu + kB) : zero;
        const LaneRandom r = row_random(a.seed, u, a.event, tile, lane);
        bool clamped = false;
        int zA[4], zB[4];
        const float inv_now = read_scale(a, 0, a.eps, a.inv_eps).inv_now;
        const uint64_t cA = round_float4<BITS>(xA, r.a0, r.a1, inv_now, zA, clamped);
        const uint64_t cB = round_float4<BITS>(xB, r.b0, r.b1, inv_now, zB, clamped);
        uint8_t *pub = a.ring + a.slot_now * ((uint64_t)a.n * a.row_bytes) + u * a.row_bytes;
        if (inA) store_code<BITS>(pub, kA / 4, cA);
        if (inB) store_code<BITS>(pub, kB / 4, cB);
        report(a.counters, 0, clamped);
    }
    if (pend) {
        if (inA) stg_nt(xu + kA, ldg_nt(wu + kA));
        if (inB) stg_nt(xu + kB, ldg_nt(wu + kB));
    }
}

// Stateless codec kernels (thread = 8 consecutive coordinates = one Philox call).
template <int BITS>
__global__ __launch_bounds__(256) void quantize_kernel(const float *__restrict__ x, uint64_t d, float inv_eps,
                                                       uint64_t seed, uint32_t node, uint32_t event,
                                                       uint8_t *__restrict__ codes, DeviceCounters *counters) {
    const uint64_t g = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    bool clamped = false;
    if (g * 8 < d) {
        const Words4 w = stream(seed, TAG_SR, 0, node, event, g);
        const f4 lo = *(const f4 *)(x + g * 8), hi = *(const f4 *)(x + g * 8 + 4);
        int z[4];
        store_code<BITS>(codes, 2 * g, round_float4<BITS>(lo, w.w0, w.w1, inv_eps, z, clamped));
        store_code<BITS>(codes, 2 * g + 1, round_float4<BITS>(hi, w.w2, w.w3, inv_eps, z, clamped));
    }
    if (counters) report(counters, 0, clamped);
}

template <int BITS>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint8_t *__restrict__ codes,
                                                         const float *__restrict__ key, uint64_t d, float eps,
                                                         float inv_eps, float *__restrict__ out) {
    const uint64_t f = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (f * 4 >= d) return;
    constexpr uint32_t MASK = (uint32_t)((1ull << BITS) - 1);
    const uint64_t c = load_code<BITS>(codes, f);
    const f4 kv = *(const f4 *)(key + f * 4);
    const float k[4] = {kv.x, kv.y, kv.z, kv.w};
    float o[4];
    bool clamped = false;
#pragma unroll
    for (int m = 0; m < 4; ++m)
        o[m] = (float)decode_near<BITS>((uint32_t)(c >> (m * BITS)) & MASK, key_cell(k[m], inv_eps, clamped)) * eps;
    *(f4 *)(out + f * 4) = f4{o[0], o[1], o[2], o[3]};
}

static dim3 tile_grid(uint64_t d, uint32_t rows) {
    const uint64_t tiles = (d + TILE - 1) / TILE;
    return dim3((unsigned)((tiles + WAVES - 1) / WAVES), rows, 1);
}

template <int BITS>
static void launch_pairs_bits(const GossipArgs &a, int delta_mode, int stale_mode, dim3 grid, hipStream_t st) {
#define SWARM_CASE(D, S)                                                                      \
    if (delta_mode == D && stale_mode == S) {                                                 \
        gossip_pairs_kernel<BITS, D, S><<<grid, WAVES * 64, 0, st>>>(a);                      \
        return;                                                                               \
    }
    if (stale_mode == 1 && !a.pair_linf) {   // both reads stale: one grid row per node
        const dim3 g2(grid.x, 2 * grid.y, 1);
        if (delta_mode == 0) gossip_nodes_kernel<BITS, 0><<<g2, WAVES * 64, 0, st>>>(a);
        else if (delta_mode == 1) gossip_nodes_kernel<BITS, 1><<<g2, WAVES * 64, 0, st>>>(a);
        else gossip_nodes_kernel<BITS, 2><<<g2, WAVES * 64, 0, st>>>(a);
        return;
    }
    SWARM_CASE(0, 0) SWARM_CASE(0, 1) SWARM_CASE(0, 2) SWARM_CASE(0, 3)
    SWARM_CASE(1, 0) SWARM_CASE(1, 1) SWARM_CASE(1, 2) SWARM_CASE(1, 3)
    SWARM_CASE(2, 0) SWARM_CASE(2, 1) SWARM_CASE(2, 2) SWARM_CASE(2, 3)
#undef SWARM_CASE
}

hipError_t launch_gossip_pairs(const GossipArgs &a, uint32_t bits, int delta_mode, int stale_mode,
                               uint32_t npairs, hipStream_t st) {
    if (npairs == 0) return hipSuccess;
    if (bits == 0) {
        const dim3 grid((unsigned)((a.d / 4 + WAVES * 64 - 1) / (WAVES * 64)), npairs, 1);
        if (delta_mode == 0) average_pairs_kernel<0><<<grid, WAVES * 64, 0, st>>>(a);
        else if (delta_mode == 1) average_pairs_kernel<1><<<grid, WAVES * 64, 0, st>>>(a);
        else average_pairs_kernel<2><<<grid, WAVES * 64, 0, st>>>(a);
        return hipGetLastError();
    }
    const dim3 grid = tile_grid(a.d, npairs);
    switch (bits) {
        case 2: launch_pairs_bits<2>(a, delta_mode, stale_mode, grid, st); break;
        case 4: launch_pairs_bits<4>(a, delta_mode, stale_mode, grid, st); break;
        case 8: launch_pairs_bits<8>(a, delta_mode, stale_mode, grid, st); break;
        case 16: launch_pairs_bits<16>(a, delta_mode, stale_mode, grid, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_gossip_singles(const GossipArgs &a, uint32_t bits, uint32_t nsingles, hipStream_t st) {
    if (nsingles == 0) return hipSuccess;
    const dim3 grid = tile_grid(a.d, nsingles);
    switch (bits) {
        case 0: gossip_singles_kernel<0><<<grid, WAVES * 64, 0, st>>>(a); break;
        case 2: gossip_singles_kernel<2><<<grid, WAVES * 64, 0, st>>>(a); break;
        case 4: gossip_singles_kernel<4><<<grid, WAVES * 64, 0, st>>>(a); break;
        case 8: gossip_singles_kernel<8><<<grid, WAVES * 64, 0, st>>>(a); break;
        case 16: gossip_singles_kernel<16><<<grid, WAVES * 64, 0, st>>>(a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_quantize(const float *x, uint64_t d, float eps, float inv_eps, uint32_t bits, uint64_t seed,
                           uint32_t node, uint32_t event, uint8_t *codes, DeviceCounters *counters,
                           hipStream_t st) {
    (void)eps;
    const unsigned blocks = (unsigned)((d / 8 + 255) / 256);
    switch (bits) {
        case 2: quantize_kernel<2><<<blocks, 256, 0, st>>>(x, d, inv_eps, seed, node, event, codes, counters); break;
        case 4: quantize_kernel<4><<<blocks, 256, 0, st>>>(x, d, inv_eps, seed, node, event, codes, counters); break;
        case 8: quantize_kernel<8><<<blocks, 256, 0, st>>>(x, d, inv_eps, seed, node, event, codes, counters); break;
        case 16: quantize_kernel<16><<<blocks, 256, 0, st>>>(x, d, inv_eps, seed, node, event, codes, counters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_dequantize(const uint8_t *codes, const float *key, uint64_t d, float eps, float inv_eps,
                             uint32_t bits, float *out, hipStream_t st) {
    const unsigned blocks = (unsigned)((d / 4 + 255) / 256);
    switch (bits) {
        case 2: dequantize_kernel<2><<<blocks, 256, 0, st>>>(codes, key, d, eps, inv_eps, out); break;
        case 4: dequantize_kernel<4><<<blocks, 256, 0, st>>>(codes, key, d, eps, inv_eps, out); break;
        case 8: dequantize_kernel<8><<<blocks, 256, 0, st>>>(codes, key, d, eps, inv_eps, out); break;
        case 16: dequantize_kernel<16><<<blocks, 256, 0, st>>>(codes, key, d, eps, inv_eps, out); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace swarm
