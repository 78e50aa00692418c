// Reductions over the model matrix: the potential Gamma = sum_i |X_i - mu|^2 with mu the
// mean model (Section 4, "Proof Overview"), and the per-pair disagreement
// max_k |X_i[k] - X_j[k]| that decides whether a b-bit code can be decoded.
// Column sums are accumulated in float64 per thread, then staged through LDS per
// workgroup; the per-workgroup partials are summed by one last workgroup in a fixed
// order, so the result does not depend on scheduling.
#include "internal.h"
#include "quant.hpp"

namespace swarm {

typedef float f4 __attribute__((ext_vector_type(4)));
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

// Non-negative floats order like their bit patterns, so atomicMax on the bits is exact
// and order-independent.
template <bool DESC>
__global__ __launch_bounds__(RB) void pair_linf_kernel(const float *__restrict__ X, uint64_t d,
                                                       const uint32_t *__restrict__ pairs,
                                                       uint32_t *__restrict__ linf_bits) {
    __shared__ float lds[RB / 64];
    // DESC: pairs are 16-byte descriptors (node ids in the first two words), else packed id pairs
    const uint32_t ni = pairs[(DESC ? 4 : 2) * blockIdx.y], nj = pairs[(DESC ? 4 : 2) * blockIdx.y + 1];
    const uint64_t f = (uint64_t)blockIdx.x * RB + threadIdx.x;
    float m = 0.f;
    if (f * 4 < d) {
        const f4 a = *(const f4 *)(X + (uint64_t)ni * d + f * 4), b = *(const f4 *)(X + (uint64_t)nj * d + f * 4);
        m = fmaxf(fmaxf(fabsf(a.x - b.x), fabsf(a.y - b.y)), fmaxf(fabsf(a.z - b.z), fabsf(a.w - b.w)));
    }
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < RB / 64; ++w) m = fmaxf(m, lds[w]);
        atomicMax(linf_bits + blockIdx.y, __float_as_uint(m));
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
    const dim3 grid((unsigned)((d / 4 + RB - 1) / RB), npairs, 1);
    pair_linf_kernel<false><<<grid, RB, 0, st>>>(X, d, pairs, linf_bits);
    return hipGetLastError();
}

hipError_t launch_pair_linf_desc(const float *X, uint64_t d, const PairDesc *pairs, uint32_t npairs,
                                 uint32_t *linf_bits, hipStream_t st) {
    if (npairs == 0) return hipSuccess;
    const dim3 grid((unsigned)((d / 4 + RB - 1) / RB), npairs, 1);
    pair_linf_kernel<true><<<grid, RB, 0, st>>>(X, d, (const uint32_t *)pairs, linf_bits);
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
