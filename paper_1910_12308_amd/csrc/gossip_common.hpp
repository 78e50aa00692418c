// Device helpers shared by the gossip kernels: tile geometry, non-temporal 128-bit accesses,
// packed code words, the per-lane random words of a row (one Philox call per 8 coordinates,
// halves swapped between neighbouring lanes), rounding of a float4 and the averaging rule.
#pragma once
#include "internal.h"
#include "philox.hpp"
#include "quant.hpp"
#include "uniform_address.hpp"

namespace swarm {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int TILE = 512;          // coordinates per wave
#ifndef SWARM_GOSSIP_WAVES
#define SWARM_GOSSIP_WAVES 8
#endif
constexpr int WAVES = SWARM_GOSSIP_WAVES;   // waves per workgroup

// Tile index of this wave as a scalar: the wave number is the same in every lane, and reading it from the
// first lane lets row bases and tile offsets live in scalar registers.
__device__ __forceinline__ uint64_t wave_tile(uint32_t waves_per_group) {
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    return (uint64_t)blockIdx.x * waves_per_group + wave;
}

__device__ __forceinline__ f4 ldg_nt(const float *p) { return __builtin_nontemporal_load((const f4 *)p); }
__device__ __forceinline__ void stg_nt(float *p, f4 v) { __builtin_nontemporal_store(v, (f4 *)p); }
// The same at `row` (the same address in every lane: a tile's first coordinate) plus the lane's offset in floats.
__device__ __forceinline__ f4 ldg_nt(const float *row, uint32_t off) {
    return __builtin_nontemporal_load((SWARM_GLOBAL const f4 *)at_bytes(uniform(row), 4u * off));
}
__device__ __forceinline__ void stg_nt(float *row, uint32_t off, f4 v) {
    __builtin_nontemporal_store(v, (SWARM_GLOBAL f4 *)at_bytes(uniform(row), 4u * off));
}
__device__ __forceinline__ uint32_t swap_with_neighbour(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true);
}

// Packed code of one float4 (4 coordinates, 4*BITS bits, coordinate m at bit m*BITS).
template <int BITS> struct CodeWord;
template <> struct CodeWord<2>  { typedef uint8_t  type; };
template <> struct CodeWord<4>  { typedef uint16_t type; };
template <> struct CodeWord<8>  { typedef uint32_t type; };
template <> struct CodeWord<16> { typedef uint64_t type; };

template <int BITS>
__device__ __forceinline__ uint64_t load_code(const uint8_t *row, uint64_t f) {
    return (uint64_t)__builtin_nontemporal_load((const typename CodeWord<BITS>::type *)(row + f * (BITS / 2)));
}
template <int BITS>
__device__ __forceinline__ void store_code(uint8_t *row, uint64_t f, uint64_t c) {
    __builtin_nontemporal_store((typename CodeWord<BITS>::type)c,
                                (typename CodeWord<BITS>::type *)(row + f * (BITS / 2)));
}
// The same for a tile's codes: `tile_codes` is the same address in every lane, f the lane's float4 within the tile.
template <int BITS>
__device__ __forceinline__ uint64_t load_tile_code(const uint8_t *tile_codes, uint32_t f) {
    typedef typename CodeWord<BITS>::type Word;
    return (uint64_t)__builtin_nontemporal_load((SWARM_GLOBAL const Word *)at_bytes(uniform(tile_codes), f * (BITS / 2)));
}
template <int BITS>
__device__ __forceinline__ void store_tile_code(uint8_t *tile_codes, uint32_t f, uint64_t c) {
    typedef typename CodeWord<BITS>::type Word;
    __builtin_nontemporal_store((Word)c, (SWARM_GLOBAL Word *)at_bytes(uniform(tile_codes), f * (BITS / 2)));
}

// The two random words of the float4 this lane holds in the tile's first half (lo*)
// and second half (hi*), for one row.
struct LaneRandom { uint32_t a0, a1, b0, b1; };

__device__ __forceinline__ LaneRandom row_random(uint64_t seed, uint32_t node, uint32_t event,
                                                 uint64_t tile, uint32_t lane) {
    const bool odd = lane & 1u;
    const uint64_t group = tile * (TILE / 8) + (lane >> 1) + (odd ? 32u : 0u);
    const Words4 w = stream(seed, TAG_SR, 0, node, event, group);
    // even lane keeps words 0,1 of group A and needs words 0,1 of group B (made by the odd lane);
    // odd lane keeps words 2,3 of group B and needs words 2,3 of group A (made by the even lane).
    const uint32_t r0 = swap_with_neighbour(odd ? w.w0 : w.w2);
    const uint32_t r1 = swap_with_neighbour(odd ? w.w1 : w.w3);
    LaneRandom out;
    out.a0 = odd ? r0 : w.w0;  out.a1 = odd ? r1 : w.w1;
    out.b0 = odd ? w.w2 : r0;  out.b1 = odd ? w.w3 : r1;
    return out;
}

template <int BITS>
__device__ __forceinline__ uint64_t round_float4(f4 x, uint32_t w_lo, uint32_t w_hi, float inv_eps,
                                                 int z[4], bool &clamped) {
    z[0] = stochastic_round(x.x, inv_eps, w_lo & 0xFFFFu, clamped);
    z[1] = stochastic_round(x.y, inv_eps, w_lo >> 16, clamped);
    z[2] = stochastic_round(x.z, inv_eps, w_hi & 0xFFFFu, clamped);
    z[3] = stochastic_round(x.w, inv_eps, w_hi >> 16, clamped);
    constexpr uint64_t MASK = (1ull << BITS) - 1;
    return ((uint64_t)z[0] & MASK) | (((uint64_t)z[1] & MASK) << BITS) |
           (((uint64_t)z[2] & MASK) << (2 * BITS)) | (((uint64_t)z[3] & MASK) << (3 * BITS));
}

// Average of own lattice point and the partner's decoded one, plus the pending update.
template <int BITS>
__device__ __forceinline__ f4 averaged(const int z_own[4], uint64_t partner_code, f4 key, f4 delta,
                                       float inv_eps, float half_eps, const int *z_true, int &fails,
                                       bool &clamped) {
    constexpr uint32_t MASK = (uint32_t)((1ull << BITS) - 1);
    const float k[4] = {key.x, key.y, key.z, key.w};
    const float dl[4] = {delta.x, delta.y, delta.z, delta.w};
    float o[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int zp = decode_near<BITS>((uint32_t)(partner_code >> (m * BITS)) & MASK,
                                         key_cell(k[m], inv_eps, clamped));
        if (z_true) fails += (zp != z_true[m]);
        o[m] = fmaf((float)(z_own[m] + zp), half_eps, dl[m]);
    }
    return f4{o[0], o[1], o[2], o[3]};
}

// The same with one lattice scale per round: the partner's code was written at eps_old, the own
// point at eps_now; far collects max |key - eps_old z_j'|, from which the next round's scale is set
// (live = false for lanes past the row end: they hold a duplicate rounded with other random words).
template <int BITS>
__device__ __forceinline__ f4 averaged_mixed(const int z_own[4], uint64_t partner_code, f4 key, f4 delta,
                                             float eps_now, float eps_old, float inv_old, const int *z_true,
                                             int &fails, bool &clamped, float &far, bool live) {
    constexpr uint32_t MASK = (uint32_t)((1ull << BITS) - 1);
    const float k[4] = {key.x, key.y, key.z, key.w};
    const float dl[4] = {delta.x, delta.y, delta.z, delta.w};
    float o[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int zp = decode_near<BITS>((uint32_t)(partner_code >> (m * BITS)) & MASK,
                                         key_cell(k[m], inv_old, clamped));
        if (z_true) fails += (zp != z_true[m]);
        const float mine = (float)z_own[m] * eps_now, theirs = (float)zp * eps_old;
        if (live) far = fmaxf(far, fabsf(k[m] - theirs));
        o[m] = (mine + theirs) * 0.5f + dl[m];
    }
    return f4{o[0], o[1], o[2], o[3]};
}

// Maximum of a non-negative float over the wave, as its bit pattern (non-negative floats order like their
// bits): row maxima through DPP, the four rows through lane reads.  The same scalar in every lane.
__device__ __forceinline__ uint32_t wave_max_bits(float v) {
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true)));
    const uint32_t b = __float_as_uint(v);
    return max(max((uint32_t)__builtin_amdgcn_readlane((int)b, 0), (uint32_t)__builtin_amdgcn_readlane((int)b, 16)),
               max((uint32_t)__builtin_amdgcn_readlane((int)b, 32), (uint32_t)__builtin_amdgcn_readlane((int)b, 48)));
}
// One lane raises *word to the wave's maximum if it is larger; the plain load only filters.
__device__ __forceinline__ void raise_to(uint32_t *word, uint32_t bits) {
    if ((threadIdx.x & 63) == 0 && bits > __atomic_load_n(word, __ATOMIC_RELAXED)) atomicMax(word, bits);
}

// Largest disagreement of the wave into the stripe of its workgroup.
__device__ __forceinline__ void report_far(uint32_t *far_bits, float far) {
    raise_to(far_bits + ((blockIdx.x + 977u * blockIdx.y) & (FAR_STRIPES - 1)), wave_max_bits(far));
}

// Scales of one read under the per-round policy (eps_slots not null), else the fixed ones.
struct ReadScale { float eps_now, inv_now, eps_old, inv_old; };
__device__ __forceinline__ ReadScale read_scale(const GossipArgs &a, uint32_t age, float eps, float inv_eps) {
    ReadScale s{eps, inv_eps, eps, inv_eps};
    if (a.eps_slots) {
        s.eps_now = a.eps_slots[a.slot_now];
        s.eps_old = a.eps_slots[(a.slot_now + a.ring_depth - age) % a.ring_depth];
        s.inv_now = 1.0f / s.eps_now;      // powers of two: exact
        s.inv_old = 1.0f / s.eps_old;
    }
    return s;
}

__device__ __forceinline__ void report(DeviceCounters *c, int fails, bool clamped) {
    if (__builtin_expect(__any(fails != 0), 0)) {
        for (int off = 32; off > 0; off >>= 1) fails += __shfl_xor(fails, off);
        if ((threadIdx.x & 63) == 0) atomicAdd(&c->decode_failures, (unsigned long long)fails);
    }
    if (__builtin_expect(__any(clamped), 0)) {
        if ((threadIdx.x & 63) == 0) atomicOr(&c->range_clamped, 1u);
    }
}

}  // namespace swarm
