// Local SGD steps for least-squares node objectives f_i(x) = 1/2 |A_i x - b_i|^2.
// Each step draws `batch` rows uniformly with replacement and uses
//   g~ = (m / batch) A_B^T (A_B w - b_B),
// an unbiased estimate of grad f_i (the paper's requirement on g~_i, Section 2).
// The work per step is two thin matrix-vector products over `batch` rows of A (about one
// flop per byte), so one workgroup per node streams those rows twice: waves take the
// row dot products (wave reduction), then every thread updates its own float4 columns.
// That form is bound by what one compute unit can pull through its cache.  Small swarms take the
// split form instead (lsq_split_kernel): a node's columns are cut into slices of 512, one workgroup
// per slice, which keeps its rows of A in registers for both products and its slice of w across all H
// steps; per step the workgroups of a node exchange only their partial residuals (batch floats each)
// through device memory, each word tagged with the launch and step it belongs to, so a reader simply
// waits until the word it needs carries the right tag (no counters, no fences, nothing to reset).  In a batch of Algorithm 1 steps the
// workgroup then runs the interaction on its slice, which is exactly one gossip tile.
#include "interact_tile.hpp"
#include "internal.h"
#include "objectives.h"
#include "philox.hpp"

namespace swarm {

constexpr int LB = 1024;

__global__ __launch_bounds__(LB) void local_lsq_kernel(const float *__restrict__ base, float *__restrict__ W,
                                                       const float *__restrict__ A, const float *__restrict__ b,
                                                       const LocalSlots slots, uint64_t d, uint32_t H,
                                                       float lr, uint32_t m_rows, uint32_t batch, uint64_t seed,
                                                       uint32_t event) {
    __shared__ uint32_t rows[LSQ_MAX_BATCH];
    __shared__ float resid[LSQ_MAX_BATCH];
    const uint32_t node = slots.nodes ? slots.nodes[blockIdx.x] : blockIdx.x;
    if (slots.steps) H = slots.steps[blockIdx.x];
    if (slots.events) event = slots.events[blockIdx.x];
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

// ---- split form ------------------------------------------------------------------------------------
constexpr int SLICE = TILE;                       // columns per workgroup: one gossip tile
constexpr int SW = 4;                             // waves per workgroup
constexpr int RMAX = LSQ_MAX_BATCH / SW;          // rows of the batch a wave holds at most
constexpr uint32_t LSQ_MAX_RESIDENT = 256;        // workgroups of one launch: they wait for one another, so all must
                                                  // be resident at once -- at most one per compute unit
constexpr uint32_t LSQ_MAX_SLICES = LSQ_MAX_RESIDENT / 2;    // a swarm has at least two nodes
constexpr unsigned long long BARRIER_TICKS = 200000000ull;   // 2 s of the 100 MHz wall clock

struct LsqSplitArgs {
    const float *base;        // n x d models the steps start from (plain local steps)
    float *W;                 // n x d live copies
    const float *A, *b;
    LocalSlots slots;         // plain local steps: which nodes
    unsigned long long *part; // exchange: [slot][step parity][slice][LSQ_MAX_BATCH] words (tag << 32 | float bits of
                              // the slice's partial residual); a reader takes a word once it carries this step's tag
    DeviceCounters *counters;
    uint64_t d, seed;
    uint32_t H, m_rows, batch, event, slices;
    uint32_t launch_tag;      // number of this launch << 8: a word's tag is launch_tag | step
    float lr;
};

// INTERACT: grid row = one step of Algorithm 1 (descriptor in ia.descs): steps from the initiator's snapshot,
// then the interaction on this slice.  Otherwise grid row = one slot of sa.slots, steps from sa.base.
template <int BITS, bool INTERACT>
__global__ __launch_bounds__(SW * 64) void lsq_split_kernel(const LsqSplitArgs sa, const InteractArgs ia) {
    __shared__ uint32_t rows[2][LSQ_MAX_BATCH];
    __shared__ float resid[LSQ_MAX_BATCH];
    __shared__ f4 gsum[SW][SLICE / 4];
    __shared__ float shares[LSQ_MAX_SLICES][LSQ_MAX_BATCH];
    __shared__ int bail;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6, slice = blockIdx.x, slot = blockIdx.y;
    SeqDesc sd{};
    uint32_t node, H = sa.H, event = sa.event;
    const float *base = sa.base;
    if (INTERACT) {
        sd = ia.descs[slot];
        node = sd.ni; H = (sd.flags >> 8) & 0xFFu; event = sd.event;
        base = ia.g.Xhat;
    } else {
        node = sa.slots.nodes ? sa.slots.nodes[slot] : slot;
        if (sa.slots.steps) H = sa.slots.steps[slot];
        if (sa.slots.events) event = sa.slots.events[slot];
    }
    const uint64_t d = sa.d;
    const uint64_t kA = (uint64_t)slice * SLICE + 4ull * lane, kB = kA + SLICE / 2;
    const bool inA = kA < d, inB = kB < d;
    const float *An = sa.A + (uint64_t)node * sa.m_rows * d, *bn = sa.b + (uint64_t)node * sa.m_rows;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const f4 hA = inA ? *(const f4 *)(base + (uint64_t)node * d + kA) : zero;
    const f4 hB = inB ? *(const f4 *)(base + (uint64_t)node * d + kB) : zero;
    f4 wA = hA, wB = hB;
    const float step = sa.lr * ((float)sa.m_rows / (float)sa.batch);
    const uint32_t batch = sa.batch, G = sa.slices;
    if (threadIdx.x == 0) bail = 0;

    // rows of step q into rows[q & 1] (threads below batch), then, after a barrier, this wave's rows of the
    // batch (s = wave, wave + 4, ...) into registers: all loads issued back to back
    auto draw_rows = [&](uint32_t q) {
        if (threadIdx.x < batch) {
            const Words4 r = stream(sa.seed, TAG_BATCH, q, node, event, threadIdx.x >> 2);
            const uint32_t word = (threadIdx.x & 3u) == 0 ? r.w0 : (threadIdx.x & 3u) == 1 ? r.w1
                                  : (threadIdx.x & 3u) == 2 ? r.w2 : r.w3;
            rows[q & 1u][threadIdx.x] = scaled_index(word, sa.m_rows);
        }
    };
    auto fetch_rows = [&](uint32_t q, f4 a[RMAX][2]) {
#pragma unroll
        for (int r = 0; r < RMAX; ++r) {
            const uint32_t s = wave + SW * r;
            a[r][0] = zero; a[r][1] = zero;
            if (s < batch) {
                const float *arow = An + (uint64_t)rows[q & 1u][s] * d;
                if (inA) a[r][0] = *(const f4 *)(arow + kA);
                if (inB) a[r][1] = *(const f4 *)(arow + kB);
            }
        }
    };
    f4 a[RMAX][2], a_next[RMAX][2];
    if (H > 0) {
        draw_rows(0);
        __syncthreads();
        fetch_rows(0, a);
    }
    for (uint32_t q = 0; q < H; ++q) {
        const uint32_t tag = sa.launch_tag | q;
        unsigned long long *mine = sa.part + (((uint64_t)slot * 2 + (q & 1u)) * G + slice) * LSQ_MAX_BATCH;
#pragma unroll
        for (int r = 0; r < RMAX; ++r) {
            const uint32_t s = wave + SW * r;
            if (s < batch) {
                float acc = 0.f;
                acc = fmaf(a[r][0].x, wA.x, acc); acc = fmaf(a[r][0].y, wA.y, acc);
                acc = fmaf(a[r][0].z, wA.z, acc); acc = fmaf(a[r][0].w, wA.w, acc);
                acc = fmaf(a[r][1].x, wB.x, acc); acc = fmaf(a[r][1].y, wB.y, acc);
                acc = fmaf(a[r][1].z, wB.z, acc); acc = fmaf(a[r][1].w, wB.w, acc);
                for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
                if (lane == 0)
                    __hip_atomic_store(mine + s, ((unsigned long long)tag << 32) | __float_as_uint(acc), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        // the next step's rows do not depend on this step's result: request them before waiting
        if (q + 1 < H) {
            draw_rows(q + 1);
            __syncthreads();
            fetch_rows(q + 1, a_next);
        }
        // the residuals: every slice's share (all polled at once, one word per thread and turn), summed in
        // slice order.  The wait is bounded, so that every wave ends whatever happens to the other workgroups.
        {
            const unsigned long long *theirs = sa.part + ((uint64_t)slot * 2 + (q & 1u)) * G * LSQ_MAX_BATCH;
            const unsigned long long t0 = wall_clock64();
            for (uint32_t p = threadIdx.x; p < batch * G; p += SW * 64) {
                const uint32_t g = p / batch, sidx = p - g * batch;
                const unsigned long long *src = theirs + (uint64_t)g * LSQ_MAX_BATCH + sidx;
                unsigned long long word = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                while ((uint32_t)(word >> 32) != tag) {
                    if (wall_clock64() - t0 > BARRIER_TICKS) { bail = 1; break; }
                    __builtin_amdgcn_s_sleep(1);
                    word = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                shares[g][sidx] = __uint_as_float((uint32_t)word);
            }
        }
        __syncthreads();
        if (bail) {
            if (threadIdx.x == 0) atomicOr(&sa.counters->barrier_timeouts, 1u);
            return;
        }
        if (threadIdx.x < batch) {
            float sum = 0.f;
            for (uint32_t g = 0; g < G; ++g) sum += shares[g][threadIdx.x];
            resid[threadIdx.x] = sum - bn[rows[q & 1u][threadIdx.x]];
        }
        __syncthreads();
        f4 gA = zero, gB = zero;
#pragma unroll
        for (int r = 0; r < RMAX; ++r) {
            const uint32_t s = wave + SW * r;
            if (s < batch) {
                const float rr = resid[s];
                gA.x = fmaf(a[r][0].x, rr, gA.x); gA.y = fmaf(a[r][0].y, rr, gA.y);
                gA.z = fmaf(a[r][0].z, rr, gA.z); gA.w = fmaf(a[r][0].w, rr, gA.w);
                gB.x = fmaf(a[r][1].x, rr, gB.x); gB.y = fmaf(a[r][1].y, rr, gB.y);
                gB.z = fmaf(a[r][1].z, rr, gB.z); gB.w = fmaf(a[r][1].w, rr, gB.w);
            }
        }
        gsum[wave][lane] = gA;
        gsum[wave][lane + 64] = gB;
        __syncthreads();
        f4 tA = gsum[0][lane], tB = gsum[0][lane + 64];
#pragma unroll
        for (int w = 1; w < SW; ++w) { tA = tA + gsum[w][lane]; tB = tB + gsum[w][lane + 64]; }
        wA.x = fmaf(-step, tA.x, wA.x); wA.y = fmaf(-step, tA.y, wA.y); wA.z = fmaf(-step, tA.z, wA.z); wA.w = fmaf(-step, tA.w, wA.w);
        wB.x = fmaf(-step, tB.x, wB.x); wB.y = fmaf(-step, tB.y, wB.y); wB.z = fmaf(-step, tB.z, wB.z); wB.w = fmaf(-step, tB.w, wB.w);
        __syncthreads();
#pragma unroll
        for (int r = 0; r < RMAX; ++r) { a[r][0] = a_next[r][0]; a[r][1] = a_next[r][1]; }
    }
    if (wave != 0) return;
    float *wrow = sa.W + (uint64_t)node * d;
    if (inA) *(f4 *)(wrow + kA) = wA;
    if (inB) *(f4 *)(wrow + kB) = wB;
    if (INTERACT) interact_tile<BITS, 3>(ia, sd, slice, lane, wA - hA, wB - hB);
}

bool lsq_split_fits(uint64_t d, uint32_t n) { return ((d + SLICE - 1) / SLICE) * n <= 256; }

hipError_t alloc_lsq(LsqObjective &o, uint64_t d, uint32_t n) {
    if (!lsq_split_fits(d, n)) return hipSuccess;
    const uint64_t slices = (d + SLICE - 1) / SLICE;
    hipError_t e;
    o.part_bytes = sizeof(unsigned long long) * n * 2 * slices * LSQ_MAX_BATCH;
    if ((e = hipMalloc((void **)&o.part, o.part_bytes)) != hipSuccess) return e;
    o.launches = 0;
    return hipMemset(o.part, 0xFF, o.part_bytes);      // no word carries the tag of a launch yet
}

// Launches are numbered so that the words one launch exchanges cannot be taken for another's; when the
// 24-bit number wraps the buffer is wiped (in stream order) before it is reused.
static hipError_t split_args(LsqSplitArgs &sa, const float *base, float *W, LsqObjective &o, const LocalSlots &slots,
                             DeviceCounters *counters, uint64_t d, uint32_t H, float lr, uint64_t seed, uint32_t event,
                             hipStream_t st) {
    sa = LsqSplitArgs{};
    o.launches = (o.launches + 1) & 0xFFFFFFu;
    if (o.launches == 0xFFFFFFu) {
        const hipError_t e = hipMemsetAsync(o.part, 0xFF, o.part_bytes, st);
        if (e != hipSuccess) return e;
        o.launches = 0;
    }
    sa.launch_tag = o.launches << 8;
    sa.base = base; sa.W = W; sa.A = o.A; sa.b = o.b; sa.slots = slots; sa.part = o.part;
    sa.counters = counters; sa.d = d; sa.seed = seed; sa.H = H; sa.m_rows = o.m_rows; sa.batch = o.batch;
    sa.event = event; sa.slices = (uint32_t)((d + SLICE - 1) / SLICE); sa.lr = lr;
    return hipSuccess;
}

hipError_t launch_local_lsq(const float *base, float *W, LsqObjective &o, const LocalSlots &slots,
                            DeviceCounters *counters, uint32_t count, uint64_t d, uint32_t H, float lr, uint64_t seed,
                            uint32_t event, hipStream_t st) {
    if (count == 0) return hipSuccess;
    if (o.part) {
        LsqSplitArgs sa;
        const hipError_t e = split_args(sa, base, W, o, slots, counters, d, H, lr, seed, event, st);
        if (e != hipSuccess) return e;
        lsq_split_kernel<0, false><<<dim3(sa.slices, count, 1), SW * 64, 0, st>>>(sa, InteractArgs{});
    } else {
        local_lsq_kernel<<<count, LB, 0, st>>>(base, W, o.A, o.b, slots, d, H, lr, o.m_rows, o.batch, seed, event);
    }
    return hipGetLastError();
}

hipError_t launch_lsq_interact(const GossipArgs &g, uint32_t bits, const SeqDesc *descs_dev, uint32_t count,
                               LsqObjective &o, float lr, hipStream_t st) {
    if (count == 0) return hipSuccess;
    if (!o.part) return hipErrorInvalidValue;
    LsqSplitArgs sa;
    const hipError_t e = split_args(sa, nullptr, const_cast<float *>(g.W), o, LocalSlots{}, g.counters, g.d, 0, lr, g.seed, 0, st);
    if (e != hipSuccess) return e;
    const InteractArgs ia{g, descs_dev, SeqDesc{}, nullptr, nullptr, 0.f, lr};
    const dim3 grid(sa.slices, count, 1);
    switch (bits) {
        case 0: lsq_split_kernel<0, true><<<grid, SW * 64, 0, st>>>(sa, ia); break;
        case 2: lsq_split_kernel<2, true><<<grid, SW * 64, 0, st>>>(sa, ia); break;
        case 4: lsq_split_kernel<4, true><<<grid, SW * 64, 0, st>>>(sa, ia); break;
        case 8: lsq_split_kernel<8, true><<<grid, SW * 64, 0, st>>>(sa, ia); break;
        case 16: lsq_split_kernel<16, true><<<grid, SW * 64, 0, st>>>(sa, ia); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

void free_lsq(LsqObjective &o) {
    if (o.part) (void)hipFree(o.part);
    o = LsqObjective{};
}

}  // namespace swarm
