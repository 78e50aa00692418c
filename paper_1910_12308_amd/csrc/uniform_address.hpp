// Global accesses written as a uniform address plus the lane's 32-bit byte offset (plus a small constant):
// the form the load and store instructions take directly (scalar base, vector offset).  The marker keeps
// the uniform part in scalar registers; without it the compiler adds the lane's offset to the base once
// and then carries 64-bit per-lane addresses -- two vector registers and two vector adds per access, and
// the registers it recycles for them make loads wait for one another.
// The pointer handed to uniform() MUST have the same value in every lane of the wave.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace swarm {

#define SWARM_GLOBAL __attribute__((address_space(1)))      // device memory, as opposed to a generic address

template <typename T>
__device__ __forceinline__ SWARM_GLOBAL T *uniform(T *p) {
    SWARM_GLOBAL T *q = (SWARM_GLOBAL T *)p;
    asm volatile("" : "+s"(q));
    return q;
}
template <typename T>
__device__ __forceinline__ SWARM_GLOBAL T *at_bytes(SWARM_GLOBAL T *p, uint32_t bytes) {
    typedef typename std::conditional<std::is_const<T>::value, const char, char>::type Byte;
    return (SWARM_GLOBAL T *)((SWARM_GLOBAL Byte *)p + bytes);
}

}  // namespace swarm
