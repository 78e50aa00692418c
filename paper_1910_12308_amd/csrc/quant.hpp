// Lattice quantizer with a decoding key (realises the Enc/Dec of Corollary 2.1):
// stochastic rounding to eps*Z, b low bits sent, decoded to the member of the
// residue class nearest to the receiver's own coordinate.
// Every float that decides an integer is one IEEE float32 operation (the library is
// built with -ffp-contract=off), so the codes are reproducible bit for bit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swarm {

constexpr float LATTICE_CLAMP = 536870912.0f;   // 2^29: keeps z_i + z_j' inside int32

// A coordinate that is not a number is flagged like an overflow and takes the lower end of the clamp
// (fmaxf returns its other operand), so that a diverged model cannot pass for a finite one unnoticed.
__device__ __forceinline__ float lattice_coord(float x, float inv_eps, bool &clamped) {
    const float t = x * inv_eps;
    clamped |= !(fabsf(t) <= LATTICE_CLAMP);
    return fminf(fmaxf(t, -LATTICE_CLAMP), LATTICE_CLAMP);
}

// z = floor(t) + [r16 + 1/2 < frac(t) 2^16]: P(up) is within 2^-17 of frac(t).
// The comparison is taken as r16 < frac(t) 2^16 - 1/2 with one fused multiply-add, whose rounding cannot
// change the decision: the scaling is a power of two; for frac(t) 2^16 >= 1/2 the difference keeps the
// operand's last bit at a smaller magnitude, so it is exact; below 1/2 it is negative however it rounds,
// and no r16 is below it.  frac(t) = t - floor(t) is exact except for tiny negative t, where the
// subtraction rounds to 1 and the hardware fraction stays one step below: either way every r16 rounds up.
__device__ __forceinline__ int stochastic_round(float x, float inv_eps, uint32_t r16, bool &clamped) {
    const float t = lattice_coord(x, inv_eps, clamped);
    const float frac = __builtin_amdgcn_fractf(t);
    const int up = (float)r16 < fmaf(frac, 65536.0f, -0.5f);
    return (int)floorf(t) + up;
}

// Lattice cell of the key (round to nearest, ties to even).
__device__ __forceinline__ int key_cell(float y, float inv_eps, bool &clamped) {
    return (int)rintf(lattice_coord(y, inv_eps, clamped));
}

// The integer congruent to c (mod 2^BITS) inside [k - 2^(BITS-1), k + 2^(BITS-1) - 1].
template <int BITS>
__device__ __forceinline__ int decode_near(uint32_t c, int k) {
    const int delta = ((int)((c - (uint32_t)k) << (32 - BITS))) >> (32 - BITS);
    return k + delta;
}

// Lattice scale for a pair at distance m (max norm): the smallest power of two >= m / (2^(b-1) - 3),
// at least 2^-100.  frexp / ldexp and one correctly rounded division: exact on both sides.
__device__ __forceinline__ float pair_scale(float m, int bits) {
    const float q = fmaxf(m, 0x1p-100f) / (float)((1 << (bits - 1)) - 3);
    int k;
    const float f = frexpf(q, &k);                 // q = f 2^k, f in [1/2, 1)
    return ldexpf(1.0f, f == 0.5f ? k - 1 : k);    // 2^ceil(log2 q)
}

}  // namespace swarm
