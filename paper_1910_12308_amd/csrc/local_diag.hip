// Local SGD steps for diagonal-quadratic node objectives
//   f_i(x) = 1/2 sum_k a_ik (x_k - c_ik)^2,   g~ = a (w - c) + sigma N(0, I)
// (appendix, definition of the local steps: the q-th gradient is taken at the base
// model minus eta times the sum of the previous ones, with a fresh sample).  All H
// steps of a coordinate stay in registers: one read of the base model, a and c, one
// write of the live copy W.  One thread owns one float4; one Philox call per step
// gives its four normals.
#include "diag_steps.hpp"

namespace swarm {

template <bool NOISE>
__global__ __launch_bounds__(256) void local_diag_kernel(const float *__restrict__ X, float *__restrict__ W,
                                                         const float *__restrict__ A, const float *__restrict__ C,
                                                         const uint32_t *__restrict__ nodes,
                                                         const uint32_t *__restrict__ steps, uint64_t d, uint32_t H,
                                                         float lr, float sigma, uint64_t seed, uint32_t event) {
    const uint64_t f = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (f * 4 >= d) return;
    const uint32_t node = nodes ? nodes[blockIdx.y] : blockIdx.y;
    const uint64_t off = (uint64_t)node * d + f * 4;
    f4 w = __builtin_nontemporal_load((const f4 *)(X + off));
    const f4 a = __builtin_nontemporal_load((const f4 *)(A + off));
    const f4 c = __builtin_nontemporal_load((const f4 *)(C + off));
    w = diag_steps<NOISE>(w, a, c, node, f, steps ? steps[node] : H, lr, sigma, seed, event);
    __builtin_nontemporal_store(w, (f4 *)(W + off));
}

hipError_t launch_local_diag(const float *X, float *W, const float *a, const float *c, const uint32_t *nodes,
                             const uint32_t *steps, uint32_t count, uint64_t d, uint32_t H, float lr, float sigma, uint64_t seed,
                             uint32_t event, hipStream_t st) {
    if (count == 0) return hipSuccess;
    const dim3 grid((unsigned)((d / 4 + 255) / 256), count, 1);
    if (sigma != 0.0f)
        local_diag_kernel<true><<<grid, 256, 0, st>>>(X, W, a, c, nodes, steps, d, H, lr, sigma, seed, event);
    else
        local_diag_kernel<false><<<grid, 256, 0, st>>>(X, W, a, c, nodes, steps, d, H, lr, sigma, seed, event);
    return hipGetLastError();
}

}  // namespace swarm
