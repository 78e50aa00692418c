// Whole round in one pass for per-coordinate objectives (diagonal quadratics): the H local steps of the
// matched nodes are taken in registers and fed straight into the quantized gossip step, so the live copy
// W never travels through memory.  Same arithmetic, in the same order, as local_diag_kernel followed by
// the gossip pass (the tile code is the shared one of round_tile.hpp with the steps as the source of the
// pending update); per pair-coordinate it reads X_i, X_j, a_i, a_j, c_i, c_j (24 B) and the two partner
// codes, and writes X_i', X_j' (8 B) and the two published codes.
#include "round_tile.hpp"

namespace swarm {

template <int BITS, int STALE, bool INPLACE, bool NOISE>
__global__ __launch_bounds__(WAVES * 64) void fused_pairs_kernel(const RoundArgs ra) {
    round_pairs_body<BITS, NOISE ? SRC_STEPS_NOISY : SRC_STEPS, STALE, INPLACE>(ra);
}

// Both reads of a pair are stale: one grid row per node (see round_node_tile).
template <int BITS, bool INPLACE, bool NOISE>
__global__ __launch_bounds__(WAVES * 64) void fused_nodes_kernel(const RoundArgs ra) {
    round_nodes_body<BITS, NOISE ? SRC_STEPS_NOISY : SRC_STEPS, INPLACE>(ra);
}

// Unmatched nodes: take the local steps and adopt the result; publish the code of the model that a
// partner would have read (the pre-step model when the apply is deferred).
template <int BITS, bool INPLACE, bool NOISE>
__global__ __launch_bounds__(WAVES * 64) void fused_singles_kernel(const RoundArgs ra) {
    round_singles_body<BITS, NOISE ? SRC_STEPS_NOISY : SRC_STEPS, INPLACE>(ra);
}

template <int BITS, bool INPLACE, bool NOISE>
static void launch_pairs_stale(const RoundArgs &ra, int stale_mode, dim3 grid, hipStream_t st) {
    switch (stale_mode) {
        case 0: fused_pairs_kernel<BITS, 0, INPLACE, NOISE><<<grid, WAVES * 64, 0, st>>>(ra); break;
        case 1:   // both reads stale: one grid row per node
            fused_nodes_kernel<BITS, INPLACE, NOISE><<<dim3(grid.x, 2 * grid.y, 1), WAVES * 64, 0, st>>>(ra);
            break;
        case 3: fused_pairs_kernel<BITS, 3, INPLACE, NOISE><<<grid, WAVES * 64, 0, st>>>(ra); break;
        default: fused_pairs_kernel<BITS, 2, INPLACE, NOISE><<<grid, WAVES * 64, 0, st>>>(ra); break;
    }
}

template <int BITS>
static void launch_bits(const RoundArgs &ra, bool inplace, bool noise, int stale_mode, uint32_t npairs,
                        uint32_t nsingles, bool singles, hipStream_t st) {
    if (!singles) {
        const dim3 grid = tile_grid(ra.g.d, npairs);
        if (inplace) { if (noise) launch_pairs_stale<BITS, true, true>(ra, stale_mode, grid, st); else launch_pairs_stale<BITS, true, false>(ra, stale_mode, grid, st); }
        else { if (noise) launch_pairs_stale<BITS, false, true>(ra, stale_mode, grid, st); else launch_pairs_stale<BITS, false, false>(ra, stale_mode, grid, st); }
    } else {
        const dim3 grid = tile_grid(ra.g.d, nsingles);
        if (inplace) { if (noise) fused_singles_kernel<BITS, true, true><<<grid, WAVES * 64, 0, st>>>(ra); else fused_singles_kernel<BITS, true, false><<<grid, WAVES * 64, 0, st>>>(ra); }
        else { if (noise) fused_singles_kernel<BITS, false, true><<<grid, WAVES * 64, 0, st>>>(ra); else fused_singles_kernel<BITS, false, false><<<grid, WAVES * 64, 0, st>>>(ra); }
    }
}

static hipError_t dispatch(const GossipArgs &g, const DiagObjective &o, uint32_t bits, bool inplace, float lr,
                           int stale_mode, uint32_t npairs, uint32_t nsingles, bool singles, hipStream_t st) {
    const RoundArgs ra{g, o.a, o.c, o.sigma, lr};
    const bool noise = o.sigma != 0.f;
    switch (bits) {
        case 2: launch_bits<2>(ra, inplace, noise, stale_mode, npairs, nsingles, singles, st); break;
        case 4: launch_bits<4>(ra, inplace, noise, stale_mode, npairs, nsingles, singles, st); break;
        case 8: launch_bits<8>(ra, inplace, noise, stale_mode, npairs, nsingles, singles, st); break;
        case 16: launch_bits<16>(ra, inplace, noise, stale_mode, npairs, nsingles, singles, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_fused_pairs(const GossipArgs &g, const DiagObjective &o, uint32_t bits, bool inplace, uint32_t H,
                              float lr, int stale_mode, uint32_t npairs, hipStream_t st) {
    (void)H;   // the step counts travel in the pair descriptors
    if (npairs == 0) return hipSuccess;
    return dispatch(g, o, bits, inplace, lr, stale_mode, npairs, 0, false, st);
}

hipError_t launch_fused_singles(const GossipArgs &g, const DiagObjective &o, uint32_t bits, bool inplace, uint32_t H,
                                float lr, uint32_t nsingles, hipStream_t st) {
    (void)H;
    if (nsingles == 0) return hipSuccess;
    return dispatch(g, o, bits, inplace, lr, 0, 0, nsingles, true, st);
}

}  // namespace swarm
