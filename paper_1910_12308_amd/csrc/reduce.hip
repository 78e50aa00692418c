// Reductions over the model matrix: the potential Gamma = sum_i |X_i - mu|^2 with mu the
// mean model (Section 4, "Proof Overview"), and the per-pair disagreement
// max_k |X_i[k] - X_j[k]| that decides whether a b-bit code can be decoded.
// Column sums are accumulated in float64 per thread, then staged through LDS per
// workgroup; the per-workgroup partials are summed by one last workgroup in a fixed
// order, so the result does not depend on scheduling.
#include <mutex>

#include "gossip_common.hpp"
#include "swarm.h"

namespace swarm {

constexpr int RB = 256;

__device__ __forceinline__ double block_sum(double v, double *lds) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) lds[wave] = v;
    __syncthreads();
    double s = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < RB / 64; ++w) s += lds[w];
    return s;   // valid in thread 0
}

// Each thread owns one float4 of columns and walks down the n rows.  With y = x - x_0
// (shift by the first row) Gamma_k = sum y^2 - (sum y)^2 / n.
__global__ __launch_bounds__(RB) void potential_kernel(const float *__restrict__ X, uint32_t n, uint64_t d,
                                                       float *__restrict__ mu, double *__restrict__ partials) {
    __shared__ double lds[RB / 64];
    const uint64_t f = (uint64_t)blockIdx.x * RB + threadIdx.x;
    double gam = 0.0;
    if (f * 4 < d) {
        const f4 x0 = *(const f4 *)(X + f * 4);
        double s1[4] = {0, 0, 0, 0}, s2[4] = {0, 0, 0, 0};
        for (uint32_t i = 1; i < n; ++i) {
            const f4 x = *(const f4 *)(X + (uint64_t)i * d + f * 4);
            const double y[4] = {(double)x.x - (double)x0.x, (double)x.y - (double)x0.y,
                                 (double)x.z - (double)x0.z, (double)x.w - (double)x0.w};
#pragma unroll
            for (int m = 0; m < 4; ++m) { s1[m] += y[m]; s2[m] += y[m] * y[m]; }
        }
        const double inv_n = 1.0 / (double)n;
#pragma unroll
        for (int m = 0; m < 4; ++m) gam += s2[m] - s1[m] * s1[m] * inv_n;
        if (mu) {
            *(f4 *)(mu + f * 4) = f4{(float)((double)x0.x + s1[0] * inv_n), (float)((double)x0.y + s1[1] * inv_n),
                                     (float)((double)x0.z + s1[2] * inv_n), (float)((double)x0.w + s1[3] * inv_n)};
        }
    }
    const double s = block_sum(gam, lds);
    if (threadIdx.x == 0) partials[blockIdx.x] = s;
}

__global__ __launch_bounds__(RB) void sum_partials_kernel(const double *__restrict__ partials, uint32_t count,
                                                          double *__restrict__ out) {
    __shared__ double lds[RB / 64];
    double v = 0.0;
    for (uint32_t i = threadIdx.x; i < count; i += RB) v += partials[i];
    const double s = block_sum(v, lds);
    if (threadIdx.x == 0) *out = s;
}

// Distance of the two models of a pair in the maximum norm: the same wave tiles and 128-bit non-temporal
// loads as the gossip pass that follows (8 bytes per pair-coordinate, nothing written but one word per
// pair).  Non-negative floats order like their bit patterns, so atomicMax on the bits is exact and
// order-independent; the waves of a workgroup meet in LDS and one lane issues at most one atomic (thousands
// of waves hitting the same word directly spend more time queueing at its memory channel than reading).
template <bool DESC>
__global__ __launch_bounds__(WAVES * 64) void pair_linf_kernel(const float *__restrict__ X, uint64_t d,
                                                               const uint32_t *__restrict__ pairs,
                                                               uint32_t *__restrict__ linf_bits) {
    __shared__ uint32_t wave_max[WAVES];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint64_t tile = wave_tile(WAVES);
    uint32_t bits = 0u;
    if (tile * TILE < d) {
    // DESC: pairs are 16-byte descriptors (node ids in the first two words), else packed id pairs
    const uint32_t ni = pairs[(DESC ? 4 : 2) * blockIdx.y], nj = pairs[(DESC ? 4 : 2) * blockIdx.y + 1];
    const uint64_t base = tile * TILE;
    const uint32_t cA = 4u * lane, cB = cA + TILE / 2;
    const bool inA = base + cA < d, inB = base + cB < d;
    const uint32_t last = (uint32_t)min((uint64_t)(TILE - 4), d - 4 - base);      // past the row end: its last float4 again
    const uint32_t oA = inA ? cA : last, oB = inB ? cB : last;
    const float *xi = X + (uint64_t)ni * d + base, *xj = X + (uint64_t)nj * d + base;
    const f4 a0 = ldg_nt(xi + oA), b0 = ldg_nt(xj + oA), a1 = ldg_nt(xi + oB), b1 = ldg_nt(xj + oB);
    const f4 e0 = a0 - b0, e1 = a1 - b1;
    const float m = fmaxf(fmaxf(fmaxf(fabsf(e0.x), fabsf(e0.y)), fmaxf(fabsf(e0.z), fabsf(e0.w))),
                          fmaxf(fmaxf(fabsf(e1.x), fabsf(e1.y)), fmaxf(fabsf(e1.z), fabsf(e1.w))));
    bits = wave_max_bits(m);
    }
    if (lane == 0) wave_max[wave] = bits;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < WAVES; ++w) bits = max(bits, wave_max[w]);
        raise_to(linf_bits + blockIdx.y * PAIR_STRIPES + (blockIdx.x & (PAIR_STRIPES - 1)), bits);
    }
}

uint32_t potential_partials(uint64_t d) { return (uint32_t)((d / 4 + RB - 1) / RB); }

hipError_t launch_potential(const float *X, uint32_t n, uint64_t d, float *mu, double *partials,
                            uint32_t npartials, double *gamma_out, hipStream_t st) {
    potential_kernel<<<npartials, RB, 0, st>>>(X, n, d, mu, partials);
    sum_partials_kernel<<<1, RB, 0, st>>>(partials, npartials, gamma_out);
    return hipGetLastError();
}

hipError_t launch_pair_linf(const float *X, uint64_t d, const uint32_t *pairs, uint32_t npairs,
                            uint32_t *linf_bits, hipStream_t st) {
    if (npairs == 0) return hipSuccess;
    const uint64_t tiles = (d + TILE - 1) / TILE;
    const dim3 grid((unsigned)((tiles + WAVES - 1) / WAVES), npairs, 1);
    pair_linf_kernel<false><<<grid, WAVES * 64, 0, st>>>(X, d, pairs, linf_bits);
    return hipGetLastError();
}

hipError_t launch_pair_linf_desc(const float *X, uint64_t d, const PairDesc *pairs, uint32_t npairs,
                                 uint32_t *linf_bits, hipStream_t st) {
    if (npairs == 0) return hipSuccess;
    const uint64_t tiles = (d + TILE - 1) / TILE;
    const dim3 grid((unsigned)((tiles + WAVES - 1) / WAVES), npairs, 1);
    pair_linf_kernel<true><<<grid, WAVES * 64, 0, st>>>(X, d, (const uint32_t *)pairs, linf_bits);
    return hipGetLastError();
}

// One lattice scale per round.  After a round: the largest |key - decoded partner| it saw sets the
// next round's scale, the smallest power of two that puts twice that distance inside the decoding
// radius, but no less than half the current scale (a round without pairs keeps the scale).
__global__ __launch_bounds__(FAR_STRIPES) void scale_close_kernel(float *eps_slots, uint32_t *state, uint32_t slot_now,
                                                                  uint32_t ring_depth, uint32_t bits, uint32_t npairs) {
    __shared__ uint32_t lds[FAR_STRIPES / 64];
    uint32_t m = state[2 + threadIdx.x];
    state[2 + threadIdx.x] = 0u;
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x != 0) return;
    for (uint32_t w = 1; w < FAR_STRIPES / 64; ++w) m = max(m, lds[w]);
    const float eps = eps_slots[slot_now];
    float next = eps;
    if (npairs) {
        next = fmaxf(pair_scale(2.0f * __uint_as_float(m), (int)bits), 0.5f * eps);
        state[1] = m;
    }
    state[0] = __float_as_uint(next);
    eps_slots[(slot_now + 1) % ring_depth] = next;
}

hipError_t launch_scale_close(float *eps_slots, uint32_t *state, uint32_t slot_now, uint32_t ring_depth,
                              uint32_t bits, uint32_t npairs, hipStream_t st) {
    scale_close_kernel<<<1, FAR_STRIPES, 0, st>>>(eps_slots, state, slot_now, ring_depth, bits, npairs);
    return hipGetLastError();
}

}  // namespace swarm

// ---- the potential without any allocation ---------------------------------------------------
// The per-workgroup partial sums of potential_kernel live in a file-scope device array instead
// of a buffer of the handle.  Every GPU holds its own copy of the array at its own address; the
// host-side name is only a stand-in, so the address is looked up once per device.
namespace {

constexpr uint32_t STATIC_PARTIALS = 1u << 17;          // 1 MiB of float64 partial sums per GPU
constexpr int MAX_DEVICES = 64;

__device__ __align__(256) double scratch[STATIC_PARTIALS];

std::mutex scratch_mutex;
double *scratch_ptr[MAX_DEVICES];                        // device address of each GPU's copy

hipError_t scratch_address(double **ptr) {
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[device]) {
        double *p = nullptr;
        e = hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        scratch_ptr[device] = p;
    }
    *ptr = scratch_ptr[device];
    return hipSuccess;
}

}  // namespace

extern "C" swarm_status swarm_potential_static(const float *X_dev, uint32_t n, uint64_t d, double *gamma_dev,
                                               float *mu_dev, void *hip_stream) {
    using namespace swarm;
    if (!X_dev || !gamma_dev || n < 1 || d == 0 || d % 4 != 0 || ((uintptr_t)X_dev & 15u) || ((uintptr_t)gamma_dev & 7u) ||
        (mu_dev && ((uintptr_t)mu_dev & 15u))) {
        set_global_error("potential (static scratch): null or misaligned pointer, n = 0, or d not a positive multiple of 4");
        return SWARM_EINVAL;
    }
    if ((d / 4 + RB - 1) / RB > STATIC_PARTIALS) {
        set_global_error("potential (static scratch): d exceeds 134217728 coordinates");
        return SWARM_EINVAL;
    }
    double *partials = nullptr;
    hipError_t e = scratch_address(&partials);
    if (e == hipSuccess)
        e = launch_potential(X_dev, n, d, mu_dev, partials, potential_partials(d), gamma_dev, (hipStream_t)hip_stream);
    if (e != hipSuccess) {
        set_global_error(hipGetErrorString(e));
        return SWARM_EDEVICE;
    }
    return SWARM_OK;
}
