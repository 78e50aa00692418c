// Local SGD steps for least-squares node objectives f_i(x) = 1/2 |A_i x - b_i|^2.
// Each step draws `batch` rows uniformly with replacement and uses
//   g~ = (m / batch) A_B^T (A_B w - b_B),
// an unbiased estimate of grad f_i (the paper's requirement on g~_i, Section 2).
// The work per step is two thin matrix-vector products over `batch` rows of A (about one
// flop per byte), so one workgroup per node streams those rows twice: waves take the
// row dot products (wave reduction), then every thread updates its own float4 columns.
#include "objectives.h"
#include "philox.hpp"

namespace swarm {

typedef float f4 __attribute__((ext_vector_type(4)));
constexpr int LB = 1024;

__global__ __launch_bounds__(LB) void local_lsq_kernel(const float *__restrict__ base, float *__restrict__ W,
                                                       const float *__restrict__ A, const float *__restrict__ b,
                                                       const uint32_t *__restrict__ nodes,
                                                       const uint32_t *__restrict__ steps, uint64_t d, uint32_t H,
                                                       float lr, uint32_t m_rows, uint32_t batch, uint64_t seed,
                                                       uint32_t event) {
    __shared__ uint32_t rows[LSQ_MAX_BATCH];
    __shared__ float resid[LSQ_MAX_BATCH];
    const uint32_t node = nodes ? nodes[blockIdx.x] : blockIdx.x;
    if (steps) H = steps[node];
    const float *An = A + (uint64_t)node * m_rows * d;
    const float *bn = b + (uint64_t)node * m_rows;
    float *wrow = W + (uint64_t)node * d;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const float step = lr * ((float)m_rows / (float)batch);
    for (uint32_t q = 0; q < H; ++q) {
        const float *src = q == 0 ? base + (uint64_t)node * d : wrow;
        if (threadIdx.x < batch) {
            const Words4 r = stream(seed, TAG_BATCH, q, node, event, threadIdx.x >> 2);
            const uint32_t word = (threadIdx.x & 3u) == 0 ? r.w0 : (threadIdx.x & 3u) == 1 ? r.w1
                                  : (threadIdx.x & 3u) == 2 ? r.w2 : r.w3;
            rows[threadIdx.x] = scaled_index(word, m_rows);
        }
        __syncthreads();
        for (uint32_t s = wave; s < batch; s += LB / 64) {
            const float *arow = An + (uint64_t)rows[s] * d;
            float acc = 0.f;
            for (uint64_t k = 4ull * lane; k < d; k += 256) {
                const f4 av = *(const f4 *)(arow + k), wv = *(const f4 *)(src + k);
                acc = fmaf(av.x, wv.x, acc); acc = fmaf(av.y, wv.y, acc);
                acc = fmaf(av.z, wv.z, acc); acc = fmaf(av.w, wv.w, acc);
            }
            for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
            if (lane == 0) resid[s] = acc - bn[rows[s]];
        }
        __syncthreads();
        for (uint64_t k = 4ull * threadIdx.x; k < d; k += 4ull * LB) {
            f4 g = {0.f, 0.f, 0.f, 0.f};
            for (uint32_t s = 0; s < batch; ++s) {
                const f4 av = *(const f4 *)(An + (uint64_t)rows[s] * d + k);
                const float r = resid[s];
                g.x = fmaf(av.x, r, g.x); g.y = fmaf(av.y, r, g.y);
                g.z = fmaf(av.z, r, g.z); g.w = fmaf(av.w, r, g.w);
            }
            f4 wv = *(const f4 *)(src + k);
            wv.x = fmaf(-step, g.x, wv.x); wv.y = fmaf(-step, g.y, wv.y);
            wv.z = fmaf(-step, g.z, wv.z); wv.w = fmaf(-step, g.w, wv.w);
            *(f4 *)(wrow + k) = wv;
        }
        __threadfence_block();
        __syncthreads();
    }
    if (H == 0)
        for (uint64_t k = 4ull * threadIdx.x; k < d; k += 4ull * LB)
            *(f4 *)(wrow + k) = *(const f4 *)(base + (uint64_t)node * d + k);
}

hipError_t launch_local_lsq(const float *base, float *W, const LsqObjective &o, const uint32_t *nodes,
                            const uint32_t *steps, uint32_t count, uint64_t d, uint32_t H, float lr, uint64_t seed, uint32_t event,
                            hipStream_t st) {
    if (count == 0) return hipSuccess;
    local_lsq_kernel<<<count, LB, 0, st>>>(base, W, o.A, o.b, nodes, steps, d, H, lr, o.m_rows, o.batch, seed, event);
    return hipGetLastError();
}

void free_lsq(LsqObjective &o) { o = LsqObjective{}; }

}  // namespace swarm
