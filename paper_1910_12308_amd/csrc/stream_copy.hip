// Plain streaming copy (one float4 per thread, non-temporal): the measured ceiling that
// the fused gossip pass is compared with, and the known-size kernel that calibrates the
// hardware byte counters.
#include "internal.h"

namespace swarm {

typedef float f4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void stream_copy_kernel(const f4 *__restrict__ src, f4 *__restrict__ dst,
                                                          uint64_t n4) {
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// The same streaming access with several concurrent streams: NR read streams are summed and
// written to NW write streams, all `n4` float4 long and `stride4` float4 apart.  HBM bandwidth on
// this part falls with the number of streams a kernel touches at once, so the gossip kernels
// (6 float read streams + 2 write streams in the one-pass round, 4 + 2 in the gossip pass) are
// compared with the copy of the same shape, not only with the 1 + 1 copy.
template <int NR, int NW>
__global__ __launch_bounds__(256) void stream_mix_kernel(const f4 *__restrict__ src, f4 *__restrict__ dst, uint64_t n4,
                                                         uint64_t stride4) {
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < NR; ++r) acc += __builtin_nontemporal_load(src + r * stride4 + i);
#pragma unroll
    for (int w = 0; w < NW; ++w) __builtin_nontemporal_store(acc + (float)w, dst + w * stride4 + i);
}

hipError_t launch_stream_mix(const void *src, void *dst, uint64_t stream_bytes, uint32_t n_read, uint32_t n_write,
                             hipStream_t st) {
    const uint64_t n4 = stream_bytes / 16;
    if (n4 == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((n4 + 255) / 256);
    const f4 *s = (const f4 *)src;
    f4 *d = (f4 *)dst;
    if (n_read == 4 && n_write == 2) stream_mix_kernel<4, 2><<<blocks, 256, 0, st>>>(s, d, n4, n4);
    else if (n_read == 6 && n_write == 2) stream_mix_kernel<6, 2><<<blocks, 256, 0, st>>>(s, d, n4, n4);
    else if (n_read == 2 && n_write == 2) stream_mix_kernel<2, 2><<<blocks, 256, 0, st>>>(s, d, n4, n4);
    else if (n_read == 3 && n_write == 1) stream_mix_kernel<3, 1><<<blocks, 256, 0, st>>>(s, d, n4, n4);
    else if (n_read == 2 && n_write == 1) stream_mix_kernel<2, 1><<<blocks, 256, 0, st>>>(s, d, n4, n4);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_stream_copy(const void *src, void *dst, uint64_t nbytes, hipStream_t st) {
    const uint64_t n4 = nbytes / 16;
    if (n4 == 0) return hipSuccess;
    stream_copy_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, st>>>((const f4 *)src, (f4 *)dst, n4);
    return hipGetLastError();
}

}  // namespace swarm
