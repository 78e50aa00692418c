// Random maximal matching of the communication graph for one gossip round (the round
// model pairs each node with at most one neighbour per round).  Every edge e gets the
// 64-bit priority (philox word << 32) | e; the result is the greedy matching that scans
// edges by increasing priority, computed in parallel: an edge joins when its priority
// is the minimum over all live edges at both endpoints, matched endpoints retire their
// edges, repeat.  One workgroup; node state lives in LDS; wave ballots drive the ordered
// compaction of the outputs (pairs by increasing edge index, unmatched nodes by index).
#include "internal.h"
#include "philox.hpp"

namespace swarm {

constexpr int MB = 1024;                      // threads of the single workgroup
constexpr uint32_t NONE = 0xFFFFFFFFu;

// Exclusive rank of this thread's flag among the workgroup's flags, in thread order,
// and the workgroup total.  wave_tot: LDS, MB/64 entries.
__device__ __forceinline__ uint32_t ordered_rank(bool flag, uint32_t *wave_tot, uint32_t &total) {
    const uint64_t mask = __ballot(flag);
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t below = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wave] = __popcll(mask);
    __syncthreads();
    uint32_t base = 0;
    total = 0;
    for (uint32_t w = 0; w < MB / 64; ++w) {
        const uint32_t t = wave_tot[w];
        if (w < wave) base += t;
        total += t;
    }
    __syncthreads();
    return base + below;
}

__global__ __launch_bounds__(MB) void matching_kernel(const uint32_t *__restrict__ edges, uint32_t n_edges,
                                                      uint32_t n, uint64_t seed, uint32_t round,
                                                      uint32_t *__restrict__ prio_hi, uint32_t *__restrict__ pairs,
                                                      uint32_t *__restrict__ singles, uint32_t *__restrict__ counts) {
    __shared__ unsigned long long node_min[MATCHING_MAX_NODES];
    __shared__ uint32_t node_edge[MATCHING_MAX_NODES];      // edge that matched the node, or NONE
    __shared__ uint32_t wave_tot[MB / 64];
    const uint32_t tid = threadIdx.x;
    for (uint32_t v = tid; v < n; v += MB) node_edge[v] = NONE;
    for (uint32_t e = tid; e < n_edges; e += MB) prio_hi[e] = stream(seed, TAG_MATCH, 0, e, round, 0).w0;
    __syncthreads();
    while (true) {
        for (uint32_t v = tid; v < n; v += MB) node_min[v] = ~0ull;
        __syncthreads();
        int live = 0;
        for (uint32_t e = tid; e < n_edges; e += MB) {
            const uint32_t u = edges[2 * e], v = edges[2 * e + 1];
            if (node_edge[u] == NONE && node_edge[v] == NONE) {
                const unsigned long long p = ((unsigned long long)prio_hi[e] << 32) | e;
                atomicMin(&node_min[u], p);
                atomicMin(&node_min[v], p);
                live = 1;
            }
        }
        if (!__syncthreads_or(live)) break;
        uint32_t win_u[4], win_v[4], win_e[4], nwin = 0;     // winners found by this thread
        for (uint32_t e = tid; e < n_edges; e += MB) {
            const uint32_t u = edges[2 * e], v = edges[2 * e + 1];
            if (node_edge[u] == NONE && node_edge[v] == NONE) {
                const unsigned long long p = ((unsigned long long)prio_hi[e] << 32) | e;
                if (node_min[u] == p && node_min[v] == p) {
                    if (nwin < 4) { win_u[nwin] = u; win_v[nwin] = v; win_e[nwin] = e; }
                    ++nwin;
                }
            }
        }
        __syncthreads();                                      // all liveness tests done before retiring nodes
        for (uint32_t w = 0; w < (nwin < 4 ? nwin : 4); ++w) { node_edge[win_u[w]] = win_e[w]; node_edge[win_v[w]] = win_e[w]; }
        __syncthreads();                                      // winners beyond 4 per thread wait for the next sweep
    }
    // pairs in increasing edge index
    uint32_t base = 0;
    for (uint32_t e0 = 0; e0 < n_edges; e0 += MB) {
        const uint32_t e = e0 + tid;
        bool chosen = false;
        uint32_t u = 0, v = 0;
        if (e < n_edges) { u = edges[2 * e]; v = edges[2 * e + 1]; chosen = node_edge[u] == e; }
        uint32_t total;
        const uint32_t rank = ordered_rank(chosen, wave_tot, total);
        if (chosen) { pairs[2 * (base + rank)] = u; pairs[2 * (base + rank) + 1] = v; }
        base += total;
    }
    uint32_t sbase = 0;
    for (uint32_t v0 = 0; v0 < n; v0 += MB) {
        const uint32_t v = v0 + tid;
        const bool single = v < n && node_edge[v] == NONE;
        uint32_t total;
        const uint32_t rank = ordered_rank(single, wave_tot, total);
        if (single) singles[sbase + rank] = v;
        sbase += total;
    }
    if (tid == 0) { counts[0] = base; counts[1] = sbase; }
}

hipError_t launch_matching(const uint32_t *edges, uint32_t n_edges, uint32_t n, uint64_t seed, uint32_t round,
                           uint32_t *prio_scratch, uint32_t *pairs, uint32_t *singles, uint32_t *counts,
                           hipStream_t st) {
    if (n > MATCHING_MAX_NODES || n_edges > MATCHING_MAX_EDGES) return hipErrorInvalidValue;
    matching_kernel<<<1, MB, 0, st>>>(edges, n_edges, n, seed, round, prio_scratch, pairs, singles, counts);
    return hipGetLastError();
}

}  // namespace swarm
