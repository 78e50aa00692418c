// Gossip pass (Section 3, "Parallel Execution"): the round kernels whose pending local steps, if any,
// sit in the live copies W -- quantize, publish, read the partner's (possibly stale) code, decode against
// the own model, average, add W - X.  The tile code is shared with the one-pass round (round_tile.hpp);
// this file holds the kernels for pending updates read from memory, plain averaging for the identity
// quantizer, and the stateless codec.
#include "round_tile.hpp"

namespace swarm {

// DELTA: 0 = no node of the launch has pending steps, 1 = all have, 2 = per-node flags in the descriptor
// (the values of SRC_NONE, SRC_LIVE, SRC_FLAGGED).
template <int BITS, int DELTA, int STALE>
__global__ __launch_bounds__(WAVES * 64) void gossip_pairs_kernel(const RoundArgs ra) {
    round_pairs_body<BITS, DELTA, STALE, false>(ra);
}

template <int BITS, int DELTA>
__global__ __launch_bounds__(WAVES * 64) void gossip_nodes_kernel(const RoundArgs ra) {
    round_nodes_body<BITS, DELTA, false>(ra);
}

// Unmatched nodes: publish the code of X_u, then apply the node's own pending steps.
template <int BITS>
__global__ __launch_bounds__(WAVES * 64) void gossip_singles_kernel(const RoundArgs ra) {
    round_singles_body<BITS, SRC_FLAGGED, false>(ra);
}

// Q = identity (Corollary 4.2): plain pairwise averaging plus the pending update.
template <int DELTA>
__global__ __launch_bounds__(WAVES * 64) void average_pairs_kernel(const GossipArgs a) {
    const uint64_t k = ((uint64_t)blockIdx.x * (WAVES * 64) + threadIdx.x) * 4;
    if (k >= a.d) return;
    const PairDesc pd = pair_desc(a, blockIdx.y);
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

template <int BITS>
static void launch_pairs_bits(const RoundArgs &ra, int delta_mode, int stale_mode, dim3 grid, hipStream_t st) {
#define SWARM_CASE(D, S)                                                                      \
    if (delta_mode == D && stale_mode == S) {                                                 \
        gossip_pairs_kernel<BITS, D, S><<<grid, WAVES * 64, 0, st>>>(ra);                     \
        return;                                                                               \
    }
    if (stale_mode == 1 && !ra.g.pair_linf) {   // both reads stale: one grid row per node
        const dim3 g2(grid.x, 2 * grid.y, 1);
        if (delta_mode == 0) gossip_nodes_kernel<BITS, 0><<<g2, WAVES * 64, 0, st>>>(ra);
        else if (delta_mode == 1) gossip_nodes_kernel<BITS, 1><<<g2, WAVES * 64, 0, st>>>(ra);
        else gossip_nodes_kernel<BITS, 2><<<g2, WAVES * 64, 0, st>>>(ra);
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
    const RoundArgs ra{a, nullptr, nullptr, 0.f, 0.f};
    switch (bits) {
        case 2: launch_pairs_bits<2>(ra, delta_mode, stale_mode, grid, st); break;
        case 4: launch_pairs_bits<4>(ra, delta_mode, stale_mode, grid, st); break;
        case 8: launch_pairs_bits<8>(ra, delta_mode, stale_mode, grid, st); break;
        case 16: launch_pairs_bits<16>(ra, delta_mode, stale_mode, grid, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_gossip_singles(const GossipArgs &a, uint32_t bits, uint32_t nsingles, hipStream_t st) {
    if (nsingles == 0) return hipSuccess;
    const dim3 grid = tile_grid(a.d, nsingles);
    const RoundArgs ra{a, nullptr, nullptr, 0.f, 0.f};
    switch (bits) {
        case 0: gossip_singles_kernel<0><<<grid, WAVES * 64, 0, st>>>(ra); break;
        case 2: gossip_singles_kernel<2><<<grid, WAVES * 64, 0, st>>>(ra); break;
        case 4: gossip_singles_kernel<4><<<grid, WAVES * 64, 0, st>>>(ra); break;
        case 8: gossip_singles_kernel<8><<<grid, WAVES * 64, 0, st>>>(ra); break;
        case 16: gossip_singles_kernel<16><<<grid, WAVES * 64, 0, st>>>(ra); break;
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
