// Steps of Algorithm 1 (sequential model): the initiator i averages its quantized model with the
// responder j's, adds the local steps it computed at its snapshot Xhat_i, and refreshes the snapshot;
// j receives the plain average:
//     X_i' = (Q(X_i) + Q(X_j)) / 2 + (W_i - Xhat_i),   X_j' = (Q(X_i) + Q(X_j)) / 2,   Xhat_i' = X_i'.
// One grid row per interaction.  Interactions whose node sets are pairwise disjoint commute, so a
// launch may carry many of them (the paper notes that Theta(n) of these interactions can occur in
// parallel: Section 2, "The Distributed System Model"); every interaction keys its random streams
// with its own interaction number, carried in its descriptor.
// LOCAL: for the diagonal-quadratic objective the initiator's H local steps are taken in registers
// from Xhat_i (same arithmetic and order as local_diag_kernel followed by W_i - Xhat_i), and the
// live copy W is neither written nor read.
#include "interact_tile.hpp"

namespace swarm {

template <int BITS, int LOCAL>
__global__ __launch_bounds__(WAVES * 64) void interact_kernel(const InteractArgs ia) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = wave_tile(WAVES);
    if (tile * TILE >= ia.g.d) return;
    const SeqDesc sd = ia.descs ? ia.descs[blockIdx.y] : ia.one;      // uniform: one scalar load
    interact_tile<BITS, LOCAL>(ia, sd, tile, lane);
}

template <int BITS>
static void launch_local_form(const InteractArgs &ia, int local, dim3 grid, hipStream_t st) {
    if (local == 0) interact_kernel<BITS, 0><<<grid, WAVES * 64, 0, st>>>(ia);
    else if (local == 1) interact_kernel<BITS, 1><<<grid, WAVES * 64, 0, st>>>(ia);
    else interact_kernel<BITS, 2><<<grid, WAVES * 64, 0, st>>>(ia);
}

hipError_t launch_interact(const GossipArgs &a, uint32_t bits, const SeqDesc *descs_dev, SeqDesc one, uint32_t count,
                           const DiagObjective *local, float lr, hipStream_t st) {
    if (count == 0) return hipSuccess;
    const uint64_t tiles = (a.d + TILE - 1) / TILE;
    const dim3 grid((unsigned)((tiles + WAVES - 1) / WAVES), count, 1);
    InteractArgs ia{a, descs_dev, one, local ? local->a : nullptr, local ? local->c : nullptr,
                    local ? local->sigma : 0.f, lr};
    const int form = !local ? 0 : (local->sigma != 0.f ? 1 : 2);
    switch (bits) {
        case 0: launch_local_form<0>(ia, form, grid, st); break;
        case 2: launch_local_form<2>(ia, form, grid, st); break;
        case 4: launch_local_form<4>(ia, form, grid, st); break;
        case 8: launch_local_form<8>(ia, form, grid, st); break;
        case 16: launch_local_form<16>(ia, form, grid, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace swarm
