// Local SGD steps for diagonal-quadratic node objectives
//   f_i(x) = 1/2 sum_k a_ik (x_k - c_ik)^2,   g~ = a (w - c) + sigma N(0, I)
// (appendix, definition of the local steps: the q-th gradient is taken at the base
// model minus eta times the sum of the previous ones, with a fresh sample).  All H
// steps of a coordinate stay in registers: one read of the base model, a and c, one
// write of the live copy W.  A wave owns a 512-coordinate tile of one node's row; a lane
// holds float4 number l and l + 64 of it (two coalesced 1 KiB accesses per array).
#include "diag_steps.hpp"

namespace swarm {

template <bool NOISE>
__global__ __launch_bounds__(WAVES * 64) void local_diag_kernel(const float *__restrict__ X, float *__restrict__ W,
                                                                const float *__restrict__ A, const float *__restrict__ C,
                                                                const LocalSlots slots, uint64_t d, uint32_t H,
                                                                float lr, float sigma, uint64_t seed, uint32_t event) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t tile = wave_tile(WAVES);
    if (tile * TILE >= d) return;
    const uint64_t kA = tile * TILE + 4ull * lane, kB = kA + TILE / 2;
    const bool inA = kA < d, inB = kB < d;
    const uint64_t lA = inA ? kA : d - 4, lB = inB ? kB : d - 4;   // past the row end: re-read its last float4
    const uint32_t node = slots.nodes ? slots.nodes[blockIdx.y] : blockIdx.y;
    if (slots.steps) H = slots.steps[blockIdx.y];
    if (slots.events) event = slots.events[blockIdx.y];
    const uint64_t off = (uint64_t)node * d;
    f4 wA = ldg_nt(X + off + lA), wB = ldg_nt(X + off + lB);
    const f4 aA = ldg_nt(A + off + lA), aB = ldg_nt(A + off + lB);
    const f4 cA = ldg_nt(C + off + lA), cB = ldg_nt(C + off + lB);
    diag_steps<NOISE>(wA, wB, aA, aB, cA, cB, node, tile, lane, H, lr, sigma, seed, event);
    if (inA) stg_nt(W + off + kA, wA);
    if (inB) stg_nt(W + off + kB, wB);
}

hipError_t launch_local_diag(const float *X, float *W, const float *a, const float *c, const LocalSlots &slots,
                             uint32_t count, uint64_t d, uint32_t H, float lr, float sigma, uint64_t seed,
                             uint32_t event, hipStream_t st) {
    if (count == 0) return hipSuccess;
    const uint64_t tiles = (d + TILE - 1) / TILE;
    const dim3 grid((unsigned)((tiles + WAVES - 1) / WAVES), count, 1);
    if (sigma != 0.0f)
        local_diag_kernel<true><<<grid, WAVES * 64, 0, st>>>(X, W, a, c, slots, d, H, lr, sigma, seed, event);
    else
        local_diag_kernel<false><<<grid, WAVES * 64, 0, st>>>(X, W, a, c, slots, d, H, lr, sigma, seed, event);
    return hipGetLastError();
}

}  // namespace swarm
