// Local SGD steps for the two-layer perceptron objective (in -> hid -> out, ReLU,
// softmax cross-entropy averaged over the batch) on a synthetic Gaussian mixture.
// Every node has its own weights, so each step is a *grouped* problem: one launch per
// GEMM covers all nodes (a one-dimensional grid over (node, tile), numbered so that a node's
// tiles run on one die), each workgroup computing a 128x128 tile of one node's product on the
// matrix cores (v_mfma_f32_32x32x2f32, float32 in and out; or three bf16 products per term).
//
// Per step:  data (labels, features)  ->  hid = relu(x W1^T + b1)  ->  logits = hid W2^T + b2
//   -> dlogits = (softmax - onehot)/batch -> dpre = (dlogits W2) * [hid > 0]
//   -> W2 -= eta dlogits^T hid, b2 -= eta colsum(dlogits), W1 -= eta dpre^T x, b1 -= eta colsum(dpre).
// The weight updates are fused into the epilogues of the two weight-gradient GEMMs, so
// the gradients never reach memory; the hidden-layer bias update rides in the epilogue of the
// backward GEMM (the tile holds the whole batch, so its column sums are the bias gradient).
//
// Tiling: 4 waves per workgroup, each wave a 64x64 sub-tile = 2x2 MFMA blocks; K is
// consumed in slabs of 16 staged through LDS (double buffered, next slab prefetched into
// registers during the MFMAs).  A 32x32x2 MFMA takes one A and one B value per lane; lanes
// 0-31 carry one k index and lanes 32-63 another, and any pairing is valid as long as A and
// B agree, so lanes 0-31 take k 0..7 of the slab and lanes 32-63 take k 8..15: operands
// whose k runs contiguously in memory are fetched from LDS with two 128-bit reads.
#include "internal.h"
#include "uniform_address.hpp"
#include "objectives.h"
#include "philox.hpp"

namespace swarm {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int TM = 128, TN = 128, TK = 16;
constexpr int LDK = TK + 4;      // row length of a [row][k] LDS tile (keeps 16-byte alignment, spreads banks)
constexpr int LDR = TM + 4;      // row length of a [k][row] LDS tile

enum Epilogue { EPI_BIAS_RELU = 0, EPI_BIAS = 1, EPI_RELU_MASK = 2, EPI_SGD_UPDATE = 3 };

struct GemmArgs {
    const float *A, *B;          // operand bases
    float *C;                    // output base
    const float *aux;            // bias (per node), ReLU mask source (per slot) or weights to update (per node)
    const uint32_t *nodes;       // slot -> node id, or null for identity
    uint64_t strideA, strideB, strideC, strideAux;   // elements between consecutive nodes / slots
    uint32_t a_by_node, b_by_node, c_by_node, aux_by_node;
    uint32_t M, N, K, lda, ldb, ldc, ldaux;
    float lr;
    // EPI_RELU_MASK only, and only when one tile covers all rows (M <= 128): dst = src - lr * column sums of C, per node
    // (the bias gradient of the hidden layer is the column sum of the matrix this GEMM produces); null = not wanted
    const float *colsum_src;
    float *colsum_dst;
    uint64_t strideColsum;
    uint32_t tiles_n, tiles_m, groups;   // workgroups of the launch: tiles_n x tiles_m per slot, total = their product x slots
};

// Which tile a workgroup computes.  The hardware deals consecutive workgroup ids round-robin over the 8
// dies (XCDs), each with its own L2; the tiles of one node share that node's activations (and nothing
// with other nodes), so the ids are renumbered to put all tiles of a node on one die, one after the
// other: die x takes the x-th eighth of the (node, tile) list.  Ids past the end of the list do nothing.
struct Tile { const float *A, *B, *aux, *colsum_src; float *C, *colsum_dst; uint32_t m0, n0; bool valid; };
__device__ __forceinline__ Tile tile_of_id(const GemmArgs &g, uint32_t id) {
    constexpr uint32_t DIES = 8;
    const uint32_t chunk = (g.groups + DIES - 1) / DIES;
    const uint32_t q = (id % DIES) * chunk + id / DIES;
    Tile t{};
    t.valid = id / DIES < chunk && q < g.groups;
    if (!t.valid) return t;
    const uint32_t per_slot = g.tiles_n * g.tiles_m, r = q % per_slot;
    const uint32_t slot = q / per_slot, node = g.nodes ? g.nodes[slot] : slot;
    t.A = g.A + (g.a_by_node ? node : slot) * g.strideA;
    t.B = g.B + (g.b_by_node ? node : slot) * g.strideB;
    t.C = g.C + (g.c_by_node ? node : slot) * g.strideC;
    t.aux = g.aux + (g.aux_by_node ? node : slot) * g.strideAux;
    t.colsum_src = g.colsum_dst ? g.colsum_src + node * g.strideColsum : nullptr;
    t.colsum_dst = g.colsum_dst ? g.colsum_dst + node * g.strideColsum : nullptr;
    t.m0 = (r / g.tiles_n) * TM;
    t.n0 = (r % g.tiles_n) * TN;
    return t;
}

// Load a 128 x 16 slab of an operand whose k index is contiguous in memory: P[row * ld + k].
__device__ __forceinline__ void fetch_kc(const float *P, uint32_t ld, uint32_t row0, uint32_t rows, uint32_t k0,
                                         f4 r[2]) {
    const uint32_t t = threadIdx.x;
    SWARM_GLOBAL const float *base = (SWARM_GLOBAL const float *)(P + k0);   // measured: no gain from the marker here
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        // rows past the matrix edge re-read its last row: they only feed outputs that are never stored
        const uint32_t row = min(row0 + (t >> 2) + 64 * i, rows - 1);
        r[i] = *(SWARM_GLOBAL const f4 *)at_bytes(base, 4 * (row * ld + 4 * (t & 3)));
    }
}
__device__ __forceinline__ void stash_kc(float *lds, const f4 r[2]) {
    const uint32_t t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 2; ++i) *(f4 *)(lds + ((t >> 2) + 64 * i) * LDK + 4 * (t & 3)) = r[i];
}
// Load a 16 x 128 slab of an operand whose row (m or n) index is contiguous: P[k * ld + row].
// A thread's k is k0 + (t >> 5) + 8 i = k0 + 2 wave + 8 i (uniform) + the lane's half.
__device__ __forceinline__ void fetch_rc(const float *P, uint32_t ld, uint32_t row0, uint32_t rows, uint32_t k0,
                                         uint32_t wave, f4 r[2]) {
    const uint32_t t = threadIdx.x, row = min(row0 + 4 * (t & 31), rows - 4);
    const uint32_t lane_bytes = 4 * (((t >> 5) & 1u) * ld + row);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        SWARM_GLOBAL const float *base = uniform(P + (uint64_t)(k0 + 2 * wave + 8 * i) * ld);
        r[i] = *(SWARM_GLOBAL const f4 *)at_bytes(base, lane_bytes);
    }
}
__device__ __forceinline__ void stash_rc(float *lds, const f4 r[2]) {
    const uint32_t t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 2; ++i) *(f4 *)(lds + ((t >> 5) + 8 * i) * LDR + 4 * (t & 31)) = r[i];
}

// The 8 operand values of this lane for one 32-row MFMA block: rows row0 + (lane % 32), k run (lane / 32) * 8 .. +7.
template <bool KC>
__device__ __forceinline__ void operand(const float *lds, uint32_t row, uint32_t half, float v[8]) {
    if (KC) {
        const f4 lo = *(const f4 *)(lds + row * LDK + 8 * half), hi = *(const f4 *)(lds + row * LDK + 8 * half + 4);
        v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
    } else {
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) v[kk] = lds[(8 * half + kk) * LDR + row];
    }
}

// Epilogues that need a tile of another matrix (the weights to update, the ReLU mask source) request it
// during the K loop, so that its HBM latency hides behind the MFMAs instead of serialising compute phase
// and memory phase.  The 64 values a lane needs are requested in eight parts, a few after the operand
// fetch of each of the first iterations: loads return in order, so a request for the whole tile ahead
// of the loop would hold back every operand slab behind it until the tile has arrived (and leave memory
// idle for the rest of the loop).  Tiles that lie wholly inside the matrix (all of them when M and N are
// multiples of 128) take straight-line loads and stores; the guarded path serves ragged edges.
struct AuxPos { const float *aux; uint32_t m0, n0, wm, wn, half, r32; bool full_tile; };
constexpr int AUX_PARTS = 8;     // part c = 4 mi + (v / 4): four consecutive rows, both column blocks

// Row group `part` (0..7) of the lane's values into the registers of row group DEST.  The caller passes
// part == DEST; the addresses are computed from the run-time value, so that they are formed when the
// part is requested (one uniform base, the lane's 32-bit offset, small constants) and not, for all
// 64 values, ahead of the loop that spreads the requests.
template <int EPI, int DEST>
__device__ __forceinline__ void prefetch_aux_rows(const GemmArgs &g, const AuxPos p, uint32_t part, float pre[2][2][16]) {
    constexpr int mi = DEST >> 2, vq = DEST & 3;
    const uint32_t row0 = p.m0 + p.wm + 32 * (part >> 2) + 8 * (part & 3u);            // uniform
    if (p.full_tile) {
        const uint32_t lane_bytes = 4 * (4 * p.half * g.ldaux + p.r32);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            SWARM_GLOBAL const float *row = uniform(p.aux + (uint64_t)(row0 + j) * g.ldaux + p.n0 + p.wn);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                SWARM_GLOBAL const float *src = at_bytes(row + 32 * ni, lane_bytes);
                // weights about to be replaced are touched once: keep them out of the way of the cached activations
                pre[mi][ni][4 * vq + j] = EPI == EPI_SGD_UPDATE ? __builtin_nontemporal_load(src) : *src;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const uint32_t n = p.n0 + p.wn + 32 * ni + p.r32, m = row0 + 4 * p.half + j;
                pre[mi][ni][4 * vq + j] = (n < g.N && m < g.M) ? p.aux[(uint64_t)m * g.ldaux + n] : 0.f;
            }
    }
}
// The K loops below are unrolled over the parts, so that each part's registers are fixed; the run-time
// copy of the part number keeps the address arithmetic inside the iteration that uses it.
__device__ __forceinline__ uint32_t at_run_time(uint32_t part) {
    asm volatile("" : "+s"(part));
    return part;
}
template <int PART> struct Part { static constexpr int value = PART; };
// Parts [FIRST, AUX_PARTS) for first <= FIRST: what a K loop of `first` iterations has not requested.
template <int EPI, int FIRST = 0>
__device__ __forceinline__ void prefetch_aux_rest(const GemmArgs &g, const AuxPos p, uint32_t first, float pre[2][2][16]) {
    if (!(EPI == EPI_RELU_MASK || EPI == EPI_SGD_UPDATE)) return;
    if constexpr (FIRST < AUX_PARTS) {
        if (first <= FIRST) prefetch_aux_rows<EPI, FIRST>(g, p, at_run_time(FIRST), pre);
        prefetch_aux_rest<EPI, FIRST + 1>(g, p, first, pre);
    }
}

// Accumulator layout of a 32x32 block (every 32x32 MFMA shape): register v of lane l holds row
// 8*(v/4) + 4*(l/32) + v%4, column l%32.
// LATE: the tile of the other matrix was not requested ahead of the K loop and is read here.
// scratch: 128 floats of LDS that nothing else uses any more (column sums, when the tile asks for them).
template <int EPI, bool LATE = false>
__device__ __forceinline__ void epilogue(const GemmArgs &g, const Tile &t, f16v acc[2][2], uint32_t wm, uint32_t wn,
                                         uint32_t half, uint32_t r32, bool full_tile, float pre[2][2][16], float *scratch) {
    float *C = t.C;
    const float *aux = t.aux;
    const uint32_t m0 = t.m0, n0 = t.n0;
    if (LATE) prefetch_aux_rest<EPI>(g, AuxPos{aux, m0, n0, wm, wn, half, r32, full_tile}, 0, pre);
    float colsum[2] = {0.f, 0.f};
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const uint32_t n = n0 + wn + 32 * ni + r32;
            const uint32_t mb = m0 + wm + 32 * mi + 4 * half;
            float bias = 0.f;
            if ((EPI == EPI_BIAS_RELU || EPI == EPI_BIAS) && n < g.N) bias = aux[n];
            float out[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float c = acc[mi][ni][v];
                if (EPI == EPI_BIAS_RELU) c = fmaxf(c + bias, 0.f);
                if (EPI == EPI_BIAS) c = c + bias;
                if (EPI == EPI_RELU_MASK) c = pre[mi][ni][v] > 0.f ? c : 0.f;
                if (EPI == EPI_SGD_UPDATE) c = fmaf(-g.lr, c, pre[mi][ni][v]);
                out[v] = c;
                if (EPI == EPI_RELU_MASK && (full_tile || mb + 8 * (v >> 2) + (v & 3) < g.M)) colsum[ni] += c;
            }
            if (full_tile) {
                const uint32_t lane_bytes = 4 * (4 * half * g.ldc + r32);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    SWARM_GLOBAL float *row =
                        uniform(C + (uint64_t)(m0 + wm + 32 * mi + 8 * (v >> 2) + (v & 3)) * g.ldc + n0 + wn + 32 * ni);
                    SWARM_GLOBAL float *dst = at_bytes(row, lane_bytes);
                    if (EPI == EPI_SGD_UPDATE) __builtin_nontemporal_store(out[v], dst); else *dst = out[v];
                }
            } else if (n < g.N) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const uint32_t m = mb + 8 * (v >> 2) + (v & 3);
                    if (m < g.M) C[(uint64_t)m * g.ldc + n] = out[v];
                }
            }
        }
    if (EPI == EPI_RELU_MASK && t.colsum_dst) {          // uniform: every wave of the workgroup takes this path
        // a column's 128 rows sit in the two halves of a wave and in the two waves with the same wn
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) colsum[ni] += __shfl_xor(colsum[ni], 32);
        if (wm != 0 && half == 0) {
            scratch[wn + r32] = colsum[0];
            scratch[wn + 32 + r32] = colsum[1];
        }
        __syncthreads();
        if (wm == 0 && half == 0) {
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const uint32_t n = n0 + wn + 32 * ni + r32;
                if (n < g.N) t.colsum_dst[n] = fmaf(-g.lr, colsum[ni] + scratch[wn + 32 * ni + r32], t.colsum_src[n]);
            }
        }
    }
}

// C (M x N) = op(A) op(B) with A_KC: A stored [m][k] else [k][m]; B_KC: B stored [n][k] else [k][n].
template <bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(256, 2) void mlp_gemm_kernel(const GemmArgs g) {
    constexpr int A_TILE = A_KC ? TM * LDK : TK * LDR, B_TILE = B_KC ? TN * LDK : TK * LDR;
    __shared__ __attribute__((aligned(16))) float lds_a[2][A_TILE];
    __shared__ __attribute__((aligned(16))) float lds_b[2][B_TILE];
    const uint32_t lane = threadIdx.x & 63u, half = lane >> 5, r32 = lane & 31u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // scalar: bases stay uniform
    const uint32_t wm = (wave >> 1) * 64, wn = (wave & 1u) * 64;
    const uint32_t slabs = g.K / TK;

    f4 ra[2], rb[2];
    auto fetch = [&](const Tile &t, uint32_t k0) {
        if (A_KC) fetch_kc(t.A, g.lda, t.m0, g.M, k0, ra); else fetch_rc(t.A, g.lda, t.m0, g.M, k0, wave, ra);
        if (B_KC) fetch_kc(t.B, g.ldb, t.n0, g.N, k0, rb); else fetch_rc(t.B, g.ldb, t.n0, g.N, k0, wave, rb);
    };
    auto stash = [&](int buf) {
        if (A_KC) stash_kc(lds_a[buf], ra); else stash_rc(lds_a[buf], ra);
        if (B_KC) stash_kc(lds_b[buf], rb); else stash_rc(lds_b[buf], rb);
    };

    const Tile t = tile_of_id(g, blockIdx.x);
    if (!t.valid) return;
    fetch(t, 0);
    f16v acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    const bool full_tile = t.m0 + TM <= g.M && t.n0 + TN <= g.N;
    float pre[2][2][16];
    const AuxPos aux_pos{t.aux, t.m0, t.n0, wm, wn, half, r32, full_tile};

    stash(0);
    __syncthreads();
    // iteration s of the K loop (s % 8 == TURN); the first four also request two parts of the other tile each,
    // which leaves the rest of even the shortest K loop (K = 128: eight iterations) to cover their latency
    auto iteration = [&](uint32_t s, auto turn) {
        constexpr int TURN = decltype(turn)::value, cur = TURN & 1;
        if (s + 1 < slabs) fetch(t, (s + 1) * TK);
        if constexpr ((EPI == EPI_RELU_MASK || EPI == EPI_SGD_UPDATE) && 2 * TURN + 1 < AUX_PARTS)
            if (s < AUX_PARTS / 2) {
                prefetch_aux_rows<EPI, 2 * TURN>(g, aux_pos, at_run_time(2 * TURN), pre);
                prefetch_aux_rows<EPI, 2 * TURN + 1>(g, aux_pos, at_run_time(2 * TURN + 1), pre);
            }
        float a[2][8], b[2][8];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) operand<A_KC>(lds_a[cur], wm + 32 * mi + r32, half, a[mi]);
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) operand<B_KC>(lds_b[cur], wn + 32 * ni + r32, half, b[ni]);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi][kk], b[ni][kk], acc[mi][ni], 0, 0, 0);
        if (s + 1 < slabs) stash(cur ^ 1);
        __syncthreads();
    };
    for (uint32_t s = 0; s < slabs; s += AUX_PARTS) {
        iteration(s, Part<0>{});
        if (s + 1 < slabs) iteration(s + 1, Part<1>{});
        if (s + 2 < slabs) iteration(s + 2, Part<2>{});
        if (s + 3 < slabs) iteration(s + 3, Part<3>{});
        if (s + 4 < slabs) iteration(s + 4, Part<4>{});
        if (s + 5 < slabs) iteration(s + 5, Part<5>{});
        if (s + 6 < slabs) iteration(s + 6, Part<6>{});
        if (s + 7 < slabs) iteration(s + 7, Part<7>{});
    }
    prefetch_aux_rest<EPI>(g, aux_pos, 2 * slabs, pre);    // K shorter than the parts

    epilogue<EPI>(g, t, acc, wm, wn, half, r32, full_tile, pre, lds_a[0]);
}

// ---- the same GEMMs as three bf16 products -----------------------------------------------------------
// Every float32 operand x is split into hi = bf16(x) and lo = bf16(x - hi) while its slab is staged into
// LDS, and a product a b is taken as a_hi b_hi + a_hi b_lo + a_lo b_hi on the bf16 matrix cores with
// float32 accumulation (the dropped terms are below 2^-16 |a b|).  The bf16 pipes run 16 times the
// float32 rate, so even at three products per term the GEMMs stop being bound by the matrix cores and
// follow the weights' memory traffic instead.
// LDS layout of a 128 x 32 operand slab, for hi and for lo: [k / 8][row][8 bf16], 16 bytes per (octet,
// row), so that the 32x32x16 MFMA's operand (lane l: row l % 32, k = 8 (l / 32) .. + 7) is one 128-bit
// read with consecutive lanes on consecutive 16-byte words; the octet planes are padded so that the staging
// writes of k-contiguous operands are free of bank conflicts too.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

constexpr int TK3 = 32;                             // K slab of the bf16 kernels: whole 128-byte lines per operand row
constexpr int OCTS = TK3 / 8;                       // octets of k per slab
constexpr int OCT_ROWS = TM + 4;                    // rows per octet plane: successive octets a quarter of the banks
                                                    // apart, so the 8-byte staging writes of half a wave (4 rows x 4
                                                    // octets x 2 halves) cover all 64 banks once
constexpr int SLAB_WORDS = OCTS * OCT_ROWS;         // 16-byte words of one operand slab (hi or lo)

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{a, b}, bf16x2));
}
// hi and lo halves of two floats, packed (first float in the low half).
__device__ __forceinline__ void split2(float a, float b, uint32_t &hi, uint32_t &lo) {
    hi = pack_bf16(a, b);
    const float ha = __uint_as_float(hi << 16), hb = __uint_as_float(hi & 0xFFFF0000u);
    lo = pack_bf16(a - ha, b - hb);
}

// k-contiguous operand P[row * ld + k]: a thread takes 4 consecutive k of four rows.  The lane's part of
// the four addresses (row * ld + its k offset, 32 bits) is computed once per tile; per slab only the uniform
// base moves.  Rows past the matrix edge re-read its last row: they only feed outputs that are never stored.
struct LaneKc { uint32_t off[4]; };
__device__ __forceinline__ LaneKc lane_kc(uint32_t ld, uint32_t row0, uint32_t rows) {
    const uint32_t t = threadIdx.x;
    LaneKc o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o.off[i] = 4 * (min(row0 + (t >> 3) + 32 * i, rows - 1) * ld + 4 * (t & 7));   // bytes
    return o;
}
// STREAM: the operand is a weight matrix read once per launch (non-temporal), not a cached activation.
template <bool STREAM>
__device__ __forceinline__ void fetch3_kc(const float *P, const LaneKc &o, uint32_t k0, f4 r[4]) {
    SWARM_GLOBAL const float *base = (SWARM_GLOBAL const float *)(P + k0);   // measured: no gain from the marker here
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        SWARM_GLOBAL const f4 *src = (SWARM_GLOBAL const f4 *)at_bytes(base, o.off[i]);
        r[i] = STREAM ? __builtin_nontemporal_load(src) : *src;
    }
}
__device__ __forceinline__ void stash3_kc(u4 *hi, u4 *lo, const f4 r[4]) {
    const uint32_t t = threadIdx.x, oct = (t & 7) >> 1, part = t & 1;      // k = 4 (t & 7) = 8 oct + 4 part
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t row = (t >> 3) + 32 * i;
        uint32_t h0, l0, h1, l1;
        split2(r[i].x, r[i].y, h0, l0);
        split2(r[i].z, r[i].w, h1, l1);
        uint2 *ph = (uint2 *)(hi + oct * OCT_ROWS + row) + part, *pl = (uint2 *)(lo + oct * OCT_ROWS + row) + part;
        *ph = uint2{h0, h1};
        *pl = uint2{l0, l1};
    }
}
// row-contiguous operand P[k * ld + row]: a thread takes one row and the 8 k of two octets (scalar loads,
// consecutive lanes on consecutive rows), so that it writes whole 16-byte words.  The octet is the same for
// the whole wave, so each load is a uniform base plus the lane's row.
template <bool STREAM>
__device__ __forceinline__ void fetch3_rc(const float *P, uint32_t ld, uint32_t row, uint32_t wave, uint32_t k0,
                                          float r[2][8]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t oct = (wave >> 1) + 2 * i;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            SWARM_GLOBAL const float *src = at_bytes(uniform(P + (uint64_t)(k0 + 8 * oct + j) * ld), 4 * row);
            r[i][j] = STREAM ? __builtin_nontemporal_load(src) : *src;
        }
    }
}
__device__ __forceinline__ void stash3_rc(u4 *hi, u4 *lo, const float r[2][8]) {
    const uint32_t t = threadIdx.x, row = t & 127;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t oct = (t >> 7) + 2 * i;
        uint32_t h[4], l[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) split2(r[i][2 * j], r[i][2 * j + 1], h[j], l[j]);
        hi[oct * OCT_ROWS + row] = u4{h[0], h[1], h[2], h[3]};
        lo[oct * OCT_ROWS + row] = u4{l[0], l[1], l[2], l[3]};
    }
}

// Scheduling hint for one pipeline iteration: one matrix instruction, then a few vector instructions, 24
// times over (a 32x32x16 instruction keeps the matrix pipe busy for 32 cycles, a vector instruction issues
// in 4).
__device__ __forceinline__ void interleave_matrix_and_vector() {
#pragma unroll
    for (int i = 0; i < 24; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // matrix
        __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);    // vector ALU
    }
}

template <bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(256, 2) void mlp_gemm3_kernel(const GemmArgs g) {
    __shared__ u4 lds[2][4][SLAB_WORDS];            // buffer x {A hi, A lo, B hi, B lo}
    const uint32_t lane = threadIdx.x & 63u, half = lane >> 5, r32 = lane & 31u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // scalar: bases stay uniform
    const uint32_t wm = (wave >> 1) * 64, wn = (wave & 1u) * 64;
    // The weights an update needs are requested during the K loop (its few slabs come from cache, the tile
    // from memory); the ReLU mask is a cached activation and is read in the epilogue, which leaves the
    // registers to the operand pipeline.
    constexpr bool AUX_AHEAD = EPI == EPI_SGD_UPDATE;

    f16v acc[2][2];
    float pre[2][2][16];

    // Operand slabs travel two iterations ahead of their use: global memory -> registers (stage s + 2),
    // registers -> LDS as bf16 hi / lo (stage s + 1), LDS -> matrix cores (stage s).  One slab in flight per
    // workgroup does not cover the memory latency at two workgroups per compute unit.
    struct Stage { f4 ka[4], kb[4]; float ra[2][8], rb[2][8]; };
    struct Rows { LaneKc a, b; uint32_t row_a, row_b; };       // the lane's part of a tile's operand addresses
    auto rows_of = [&](const Tile &t) {
        Rows r{};
        if (A_KC) r.a = lane_kc(g.lda, t.m0, g.M); else r.row_a = min(t.m0 + (threadIdx.x & 127u), g.M - 1);
        if (B_KC) r.b = lane_kc(g.ldb, t.n0, g.N); else r.row_b = min(t.n0 + (threadIdx.x & 127u), g.N - 1);
        return r;
    };
    auto fetch = [&](const Tile &t, const Rows &rw, uint32_t k0, Stage &r) {
        // in the forward and backward products B is a weight matrix; in the updates both operands are activations
        constexpr bool B_STREAM = EPI != EPI_SGD_UPDATE;
        if (A_KC) fetch3_kc<false>(t.A, rw.a, k0, r.ka); else fetch3_rc<false>(t.A, g.lda, rw.row_a, wave, k0, r.ra);
        if (B_KC) fetch3_kc<B_STREAM>(t.B, rw.b, k0, r.kb); else fetch3_rc<B_STREAM>(t.B, g.ldb, rw.row_b, wave, k0, r.rb);
    };
    auto stash = [&](int buf, const Stage &r) {
        if (A_KC) stash3_kc(lds[buf][0], lds[buf][1], r.ka); else stash3_rc(lds[buf][0], lds[buf][1], r.ra);
        if (B_KC) stash3_kc(lds[buf][2], lds[buf][3], r.kb); else stash3_rc(lds[buf][2], lds[buf][3], r.rb);
    };
    auto clear = [&]() {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    };
    auto multiply = [&](int cur) {
#pragma unroll
        for (int ks = 0; ks < TK3 / 16; ++ks) {      // one 32x32x16 step per pair of octets
            bf16x8 ah[2], al[2], bh[2], bl[2];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const uint32_t w = (2 * ks + half) * OCT_ROWS + wm + 32 * mi + r32;
                ah[mi] = __builtin_bit_cast(bf16x8, lds[cur][0][w]);
                al[mi] = __builtin_bit_cast(bf16x8, lds[cur][1][w]);
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const uint32_t w = (2 * ks + half) * OCT_ROWS + wn + 32 * ni + r32;
                bh[ni] = __builtin_bit_cast(bf16x8, lds[cur][2][w]);
                bl[ni] = __builtin_bit_cast(bf16x8, lds[cur][3][w]);
            }
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[mi], bh[ni], acc[mi][ni], 0, 0, 0);
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[mi], bl[ni], acc[mi][ni], 0, 0, 0);
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[mi], bh[ni], acc[mi][ni], 0, 0, 0);
                }
        }
    };
    const uint32_t slabs = g.K / TK3;
    const Tile t = tile_of_id(g, blockIdx.x);
    if (!t.valid) return;
    const Rows rw = rows_of(t);
    if (AUX_AHEAD) {                                 // registers hold the weight tile: one slab ahead
        Stage next;
        fetch(t, rw, 0, next);
        clear();
        const bool full_tile = t.m0 + TM <= g.M && t.n0 + TN <= g.N;
        const AuxPos aux_pos{t.aux, t.m0, t.n0, wm, wn, half, r32, full_tile};
        stash(0, next);
        __syncthreads();
        // iteration s (s % 4 == TURN); in the first pass it also requests a quarter of the weight tile (K = 128 is
        // four iterations)
        auto iteration = [&](uint32_t s, auto turn) {
            constexpr int TURN = decltype(turn)::value, cur = TURN & 1;
            if (s + 1 < slabs) fetch(t, rw, (s + 1) * TK3, next);
            if (s < AUX_PARTS / 2) {
                prefetch_aux_rows<EPI, 2 * TURN>(g, aux_pos, at_run_time(2 * TURN), pre);
                prefetch_aux_rows<EPI, 2 * TURN + 1>(g, aux_pos, at_run_time(2 * TURN + 1), pre);
            }
            multiply(cur);
            if (s + 1 < slabs) stash(cur ^ 1, next);
            __syncthreads();
        };
        for (uint32_t s = 0; s < slabs; s += 4) {
            iteration(s, Part<0>{});
            if (s + 1 < slabs) iteration(s + 1, Part<1>{});
            if (s + 2 < slabs) iteration(s + 2, Part<2>{});
            if (s + 3 < slabs) iteration(s + 3, Part<3>{});
        }
        prefetch_aux_rest<EPI>(g, aux_pos, 2 * slabs, pre);
        epilogue<EPI, false>(g, t, acc, wm, wn, half, r32, full_tile, pre, (float *)lds[0][0]);
    } else {
        clear();
        const bool full_tile = t.m0 + TM <= g.M && t.n0 + TN <= g.N;
        Stage even, odd;                             // slab s waits in `even` when s is even, else in `odd`
        fetch(t, rw, 0, even);
        if (slabs > 1) fetch(t, rw, TK3, odd);
        stash(0, even);
        __syncthreads();
        // iteration s: request slab s + 2 into the registers slab s has just left, multiply slab s, stage slab s + 1.
        // In the steady state the conversion of slab s + 1 (vector ALU, its data arrived an iteration ago) is
        // issued between the matrix instructions of slab s, which would otherwise run one after the other
        // with the vector ALU idle, and then the other way round.
        uint32_t s = 0;
        for (; s + 3 < slabs; s += 2) {
            fetch(t, rw, (s + 2) * TK3, even);
            multiply(0);
            stash(1, odd);
            interleave_matrix_and_vector();
            __syncthreads();
            fetch(t, rw, (s + 3) * TK3, odd);
            multiply(1);
            stash(0, even);
            interleave_matrix_and_vector();
            __syncthreads();
        }
        for (; s < slabs; ++s) {                     // the last slabs: nothing left to request
            const bool to_even = (s & 1u) != 0;      // slab s + 1 waits in `even` when s is odd
            if (s + 2 < slabs) { if (to_even) fetch(t, rw, (s + 2) * TK3, odd); else fetch(t, rw, (s + 2) * TK3, even); }
            multiply(s & 1);
            if (s + 1 < slabs) { if (to_even) stash(0, even); else stash(1, odd); }
            __syncthreads();
        }
        epilogue<EPI, true>(g, t, acc, wm, wn, half, r32, full_tile, pre, (float *)lds[0][0]);
    }
}

// Labels by inverse CDF: y = #{c : cdf[c] <= u}, u = (word >> 8) 2^-24, limited to n_out - 1.
__global__ void mlp_labels_kernel(const float *__restrict__ cdf, const uint32_t *__restrict__ nodes,
                                  const uint32_t *__restrict__ events, uint32_t *__restrict__ labels, uint32_t n_out,
                                  uint32_t batch, uint64_t seed, uint32_t event, uint32_t q) {
    const uint32_t slot = blockIdx.x, node = nodes ? nodes[slot] : slot;
    if (events) event = events[slot];
    for (uint32_t s = threadIdx.x; s < batch; s += blockDim.x) {
        const Words4 w = stream(seed, TAG_LABEL, q, node, event, s >> 2);
        const uint32_t word = (s & 3u) == 0 ? w.w0 : (s & 3u) == 1 ? w.w1 : (s & 3u) == 2 ? w.w2 : w.w3;
        const float u = (float)(word >> 8) * 0x1p-24f;
        const float *row = cdf + (uint64_t)node * n_out;
        uint32_t lo = 0, hi = n_out;                      // first index with cdf > u
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (row[mid] <= u) lo = mid + 1; else hi = mid;
        }
        labels[(uint64_t)slot * batch + s] = lo < n_out ? lo : n_out - 1;
    }
}

// Features: x[s] = means[y_s] + sigma N(0, I); one Philox call per float4.
__global__ __launch_bounds__(256) void mlp_features_kernel(const float *__restrict__ means,
                                                           const uint32_t *__restrict__ nodes,
                                                           const uint32_t *__restrict__ events,
                                                           const uint32_t *__restrict__ labels, float *__restrict__ x,
                                                           uint32_t n_in, uint32_t batch, float sigma, uint64_t seed,
                                                           uint32_t event, uint32_t q) {
    const uint32_t slot = blockIdx.y, node = nodes ? nodes[slot] : slot;
    if (events) event = events[slot];
    const uint64_t f = (uint64_t)blockIdx.x * 256 + threadIdx.x;       // float4 index within the batch
    if (f * 4 >= (uint64_t)batch * n_in) return;
    const uint32_t s = (uint32_t)(f * 4 / n_in), k = (uint32_t)(f * 4 % n_in);
    const uint32_t y = labels[(uint64_t)slot * batch + s];
    const Words4 w = stream(seed, TAG_DATA, q, node, event, f);
    float z0, z1, z2, z3;
    box_muller(w.w0, w.w1, z0, z1);
    box_muller(w.w2, w.w3, z2, z3);
    const f4 mu = *(const f4 *)(means + (uint64_t)y * n_in + k);
    f4 out;
    out.x = fmaf(sigma, z0, mu.x); out.y = fmaf(sigma, z1, mu.y);
    out.z = fmaf(sigma, z2, mu.z); out.w = fmaf(sigma, z3, mu.w);
    *(f4 *)(x + ((uint64_t)slot * batch + s) * n_in + k) = out;
}

__device__ __forceinline__ float block_reduce(float v, float *lds, bool is_max) {
    for (int off = 32; off > 0; off >>= 1) {
        const float o = __shfl_xor(v, off);
        v = is_max ? fmaxf(v, o) : v + o;
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = lds[0];
    for (uint32_t w = 1; w < blockDim.x / 64; ++w) r = is_max ? fmaxf(r, lds[w]) : r + lds[w];
    return r;
}

// In place: logits row -> (softmax - onehot(y)) / batch.  Rows of up to 2048 entries stay in registers between
// the three passes (maximum, sum of exponentials, result): one read and one write of the row.
__global__ __launch_bounds__(256) void mlp_softmax_grad_kernel(float *__restrict__ logits,
                                                               const uint32_t *__restrict__ labels, uint32_t n_out,
                                                               uint32_t batch) {
    __shared__ float lds[4];
    const uint32_t slot = blockIdx.y, s = blockIdx.x;
    float *row = logits + ((uint64_t)slot * batch + s) * n_out;
    const uint32_t y = labels[(uint64_t)slot * batch + s];
    const float inv_b = 1.0f / (float)batch;
    constexpr int HELD = 8;
    if (n_out <= 256 * HELD) {
        float v[HELD];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < HELD; ++i) {
            const uint32_t c = threadIdx.x + 256 * i;
            v[i] = c < n_out ? row[c] : -INFINITY;
            mx = fmaxf(mx, v[i]);
        }
        mx = block_reduce(mx, lds, true);
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < HELD; ++i) {
            v[i] = expf(v[i] - mx);              // exp(-inf) = 0 for the entries past the row
            sum += v[i];
        }
        sum = block_reduce(sum, lds, false);
#pragma unroll
        for (int i = 0; i < HELD; ++i) {
            const uint32_t c = threadIdx.x + 256 * i;
            if (c < n_out) row[c] = (v[i] / sum - (c == y ? 1.f : 0.f)) * inv_b;
        }
        return;
    }
    float mx = -INFINITY;
    for (uint32_t c = threadIdx.x; c < n_out; c += 256) mx = fmaxf(mx, row[c]);
    mx = block_reduce(mx, lds, true);
    float sum = 0.f;
    for (uint32_t c = threadIdx.x; c < n_out; c += 256) sum += expf(row[c] - mx);
    sum = block_reduce(sum, lds, false);
    for (uint32_t c = threadIdx.x; c < n_out; c += 256)
        row[c] = (expf(row[c] - mx) / sum - (c == y ? 1.f : 0.f)) * inv_b;
}

// b_dst = b_src - lr * column sums of G (batch x width).
__global__ __launch_bounds__(256) void mlp_bias_kernel(const float *__restrict__ G, const float *__restrict__ src,
                                                       float *__restrict__ dst, const uint32_t *__restrict__ nodes,
                                                       uint32_t width, uint32_t batch, uint64_t d, uint64_t bias_off,
                                                       float lr) {
    const uint32_t slot = blockIdx.y, node = nodes ? nodes[slot] : slot;
    const uint32_t c = blockIdx.x * 256 + threadIdx.x;
    if (c >= width) return;
    const float *g = G + (uint64_t)slot * batch * width;
    float sum = 0.f;
    for (uint32_t s = 0; s < batch; ++s) sum += g[(uint64_t)s * width + c];
    dst[(uint64_t)node * d + bias_off + c] = fmaf(-lr, sum, src[(uint64_t)node * d + bias_off + c]);
}

hipError_t alloc_mlp(MlpObjective &o, uint32_t n_nodes) {
    o.n_nodes = n_nodes;
    const size_t b = o.batch;
    hipError_t e;
    if ((e = hipMalloc((void **)&o.x, sizeof(float) * n_nodes * b * o.n_in)) != hipSuccess) return e;
    if ((e = hipMalloc((void **)&o.hid, sizeof(float) * n_nodes * b * o.n_hid)) != hipSuccess) return e;
    if ((e = hipMalloc((void **)&o.dlogits, sizeof(float) * n_nodes * b * o.n_out)) != hipSuccess) return e;
    if ((e = hipMalloc((void **)&o.dhid, sizeof(float) * n_nodes * b * o.n_hid)) != hipSuccess) return e;
    if ((e = hipMalloc((void **)&o.labels, sizeof(uint32_t) * n_nodes * b)) != hipSuccess) return e;
    return hipSuccess;
}

void free_mlp(MlpObjective &o) {
    void *p[] = {o.x, o.hid, o.dlogits, o.dhid, o.labels};
    for (void *q : p) if (q) (void)hipFree(q);
    o = MlpObjective{};
}

template <bool A_KC, bool B_KC, int EPI>
static void gemm(GemmArgs g, uint32_t count, bool split, hipStream_t st) {
    g.tiles_n = (g.N + TN - 1) / TN;
    g.tiles_m = (g.M + TM - 1) / TM;
    g.groups = g.tiles_n * g.tiles_m * count;
    const dim3 grid(8 * ((g.groups + 7) / 8), 1, 1);          // a whole number of turns over the dies
    if (split) mlp_gemm3_kernel<A_KC, B_KC, EPI><<<grid, 256, 0, st>>>(g);
    else mlp_gemm_kernel<A_KC, B_KC, EPI><<<grid, 256, 0, st>>>(g);
}

hipError_t launch_local_mlp(const float *base, float *W, const MlpObjective &o, const LocalSlots &slots,
                            uint32_t count, uint32_t n, uint64_t d, uint32_t H, float lr, uint64_t seed,
                            uint32_t event, hipStream_t st) {
    (void)n;
    const uint32_t *nodes = slots.nodes;          // the number of steps is constant for this objective
    if (count == 0) return hipSuccess;
    const uint32_t I = o.n_in, Hd = o.n_hid, O = o.n_out, Bt = o.batch;
    const uint64_t off_b1 = (uint64_t)Hd * I, off_w2 = off_b1 + Hd, off_b2 = off_w2 + (uint64_t)O * Hd;
    for (uint32_t q = 0; q < H; ++q) {
        const float *src = q == 0 ? base : W;
        mlp_labels_kernel<<<count, 128, 0, st>>>(o.cdf, nodes, slots.events, o.labels, O, Bt, seed, event, q);
        mlp_features_kernel<<<dim3((unsigned)(((uint64_t)Bt * I / 4 + 255) / 256), count), 256, 0, st>>>(
            o.means, nodes, slots.events, o.labels, o.x, I, Bt, o.data_sigma, seed, event, q);
        GemmArgs g{};
        g.nodes = nodes; g.lr = lr;
        // hid = relu(x W1^T + b1):  M = batch, N = hid, K = in
        g.A = o.x; g.strideA = (uint64_t)Bt * I; g.a_by_node = 0; g.lda = I;
        g.B = src; g.strideB = d; g.b_by_node = 1; g.ldb = I;
        g.C = o.hid; g.strideC = (uint64_t)Bt * Hd; g.c_by_node = 0; g.ldc = Hd;
        g.aux = src + off_b1; g.strideAux = d; g.aux_by_node = 1; g.ldaux = 0;
        g.M = Bt; g.N = Hd; g.K = I;
        gemm<true, true, EPI_BIAS_RELU>(g, count, o.bf16x3, st);
        // logits = hid W2^T + b2:  M = batch, N = out, K = hid
        g.A = o.hid; g.strideA = (uint64_t)Bt * Hd; g.lda = Hd;
        g.B = src + off_w2; g.ldb = Hd;
        g.C = o.dlogits; g.strideC = (uint64_t)Bt * O; g.ldc = O;
        g.aux = src + off_b2;
        g.M = Bt; g.N = O; g.K = Hd;
        gemm<true, true, EPI_BIAS>(g, count, o.bf16x3, st);
        mlp_softmax_grad_kernel<<<dim3(Bt, count), 256, 0, st>>>(o.dlogits, o.labels, O, Bt);
        // dpre = (dlogits W2) * [hid > 0]:  M = batch, N = hid, K = out;  W2 stored [k][n]
        g.A = o.dlogits; g.strideA = (uint64_t)Bt * O; g.lda = O;
        g.B = src + off_w2; g.ldb = Hd;
        g.C = o.dhid; g.strideC = (uint64_t)Bt * Hd; g.ldc = Hd;
        g.aux = o.hid; g.strideAux = (uint64_t)Bt * Hd; g.aux_by_node = 0; g.ldaux = Hd;
        g.M = Bt; g.N = Hd; g.K = O;
        // b1 <- b1 - eta colsum(dpre), inside this GEMM when one tile holds the whole batch
        const bool b1_inside = Bt <= (uint32_t)TM;
        if (b1_inside) { g.colsum_src = src + off_b1; g.colsum_dst = W + off_b1; g.strideColsum = d; }
        gemm<true, false, EPI_RELU_MASK>(g, count, o.bf16x3, st);
        g.colsum_src = nullptr; g.colsum_dst = nullptr;
        // W2 <- W2 - eta dlogits^T hid:  M = out, N = hid, K = batch;  both operands stored [k][row]
        g.A = o.dlogits; g.strideA = (uint64_t)Bt * O; g.a_by_node = 0; g.lda = O;
        g.B = o.hid; g.strideB = (uint64_t)Bt * Hd; g.b_by_node = 0; g.ldb = Hd;
        g.C = W + off_w2; g.strideC = d; g.c_by_node = 1; g.ldc = Hd;
        g.aux = src + off_w2; g.strideAux = d; g.aux_by_node = 1; g.ldaux = Hd;
        g.M = O; g.N = Hd; g.K = Bt;
        gemm<false, false, EPI_SGD_UPDATE>(g, count, o.bf16x3, st);
        mlp_bias_kernel<<<dim3((O + 255) / 256, count), 256, 0, st>>>(o.dlogits, src, W, nodes, O, Bt, d, off_b2, lr);
        // W1 <- W1 - eta dpre^T x:  M = hid, N = in, K = batch
        g.A = o.dhid; g.strideA = (uint64_t)Bt * Hd; g.lda = Hd;
        g.B = o.x; g.strideB = (uint64_t)Bt * I; g.ldb = I;
        g.C = W; g.ldc = I;
        g.aux = src; g.ldaux = I;
        g.M = Hd; g.N = I; g.K = Bt;
        gemm<false, false, EPI_SGD_UPDATE>(g, count, o.bf16x3, st);
        if (!b1_inside)
            mlp_bias_kernel<<<dim3((Hd + 255) / 256, count), 256, 0, st>>>(o.dhid, src, W, nodes, Hd, Bt, d, off_b1, lr);
    }
    return hipGetLastError();
}

}  // namespace swarm
