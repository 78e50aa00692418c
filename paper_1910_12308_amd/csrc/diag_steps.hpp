// H local SGD steps of one float4 of a diagonal-quadratic objective, in registers:
//   g = a (w - c) + sigma N(0, I),  w <- w - eta g,  a fresh Gaussian sample every step
// (one Philox call per step gives the four normals of float4 number f of the node's row).
#pragma once
#include "internal.h"
#include "philox.hpp"

namespace swarm {

typedef float f4 __attribute__((ext_vector_type(4)));

template <bool NOISE>
__device__ __forceinline__ f4 diag_steps(f4 w, const f4 a, const f4 c, uint32_t node, uint64_t f, uint32_t H,
                                         float lr, float sigma, uint64_t seed, uint32_t event) {
    for (uint32_t q = 0; q < H; ++q) {
        f4 noise = {0.f, 0.f, 0.f, 0.f};
        if (NOISE) {
            const Words4 r = stream(seed, TAG_NOISE, q, node, event, f);
            float n0, n1, n2, n3;
            box_muller(r.w0, r.w1, n0, n1);
            box_muller(r.w2, r.w3, n2, n3);
            noise = f4{n0, n1, n2, n3} * sigma;
        }
        const f4 t = w - c;
        f4 g;
        g.x = fmaf(a.x, t.x, noise.x); g.y = fmaf(a.y, t.y, noise.y);
        g.z = fmaf(a.z, t.z, noise.z); g.w = fmaf(a.w, t.w, noise.w);
        w.x = fmaf(-lr, g.x, w.x); w.y = fmaf(-lr, g.y, w.y);
        w.z = fmaf(-lr, g.z, w.z); w.w = fmaf(-lr, g.w, w.w);
    }
    return w;
}

}  // namespace swarm
