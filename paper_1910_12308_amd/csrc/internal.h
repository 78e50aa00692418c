// Internal launch interfaces between the C-ABI translation unit and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swarm {

// Text returned by swarm_last_error(NULL): failures of calls that have no handle.
void set_global_error(const char *message);

// Device-side counters shared by the kernels (one per handle).
struct DeviceCounters {
    unsigned long long decode_failures;
    unsigned int range_clamped;
    unsigned int barrier_timeouts;   // a workgroup gave up waiting for the others of its node (least-squares split form)
};

// Multi-resolution registers: tiles read beyond the first plane (to 8 bits, to 16 bits), the coordinates
// in those tiles, and tiles that no level confirmed.  Kept in PREFIX_STRIPES copies that workgroups
// spread over, so that a round in which every tile escalates does not serialise on one address; the
// host adds the stripes up.
struct PrefixStats {
    unsigned long long tiles[2], coords[2], unconfirmed;
    unsigned long long written_back[2];   // Algorithm 1: coordinates whose average went back with 8 / 16 bits
    unsigned long long pad;
};
constexpr uint32_t PREFIX_STRIPES = 4096;

// One matched pair of a round.  flags: bits 0-7 = age (in rounds) of the code i reads from j,
// bits 8-15 = age of the code j reads from i, bit 16 / 17 = W_i / W_j carries unapplied steps.
// steps: bits 0-7 / 8-15 = number of local steps of i / j (used by the one-pass round).
// 16 bytes so that a workgroup fetches its pair with one scalar load.
struct PairDesc {
    uint32_t ni, nj, flags, steps;
};
// Unmatched-node entry: node id (bits 0-15) | number of local steps (bits 16-23) | pending flag.
constexpr uint32_t SINGLE_PENDING = 0x80000000u;
constexpr uint32_t SINGLE_NODE_MASK = 0xFFFFu;

struct GossipArgs {
    float *X;                 // n x d current models (updated in place)
    const float *W;           // n x d live copies
    float *Xhat;              // n x d snapshots (Algorithm 1 only), may be null
    uint8_t *ring;            // (S+1) x n x row_bytes packed codes
    const PairDesc *pairs;    // device: one per matched pair
    const uint32_t *singles;  // device: unmatched nodes (node id | SINGLE_PENDING)
    const uint32_t *pair_linf; // device: PAIR_STRIPES words per pair (same order as pairs) whose maximum is the bit
                              // pattern of max_k |X_i - X_j|, or null when the lattice scale is fixed
    const float *eps_slots;   // device: lattice scale of the codes in each ring slot (one scale per round), or
                              // null when the scale is fixed or per pair
    uint32_t *far_bits;       // device: FAR_STRIPES words, each the float bits of the largest |key - decoded
                              // partner| reported into it this round (with eps_slots); the round's maximum is
                              // their maximum
    PrefixStats *prefix_stats; // device: PREFIX_STRIPES entries (multi-resolution registers), or null
    DeviceCounters *counters;
    uint64_t d;
    uint64_t row_bytes;       // d * bits / 8
    uint64_t seed;
    uint32_t n;
    uint32_t event;           // round number (or interaction number in Algorithm 1)
    uint32_t slot_now;        // ring slot written this round
    uint32_t ring_depth;      // S + 1
    float eps, inv_eps;
};
#if defined(__HIPCC__)
// Descriptor k of the launch (k is uniform: a scalar load).  The fields are read from the first lane
// explicitly, so that everything derived from them (row bases, ring slots) provably lives in scalar
// registers.
__device__ __forceinline__ uint32_t first_lane(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ PairDesc pair_desc(const GossipArgs &g, uint32_t k) {
    const PairDesc pd = g.pairs[k];
    return PairDesc{first_lane(pd.ni), first_lane(pd.nj), first_lane(pd.flags), first_lane(pd.steps)};
}
__device__ __forceinline__ uint32_t single_desc(const GossipArgs &g, uint32_t k) { return first_lane(g.singles[k]); }
#endif

// delta_mode: 0 = no node of these pairs has pending steps, 1 = all have, 2 = per-pair flags.
// stale_mode: 0 = all reads fresh, 1 = all stale, 2 = per-pair flags, 3 = in every pair only the
// first node's read is stale.
hipError_t launch_gossip_pairs(const GossipArgs &a, uint32_t bits, int delta_mode, int stale_mode,
                               uint32_t npairs, hipStream_t st);
hipError_t launch_gossip_singles(const GossipArgs &a, uint32_t bits, uint32_t nsingles, hipStream_t st);
// One interaction of Algorithm 1: initiator ni, responder nj, the interaction number that keys its
// random streams, and flags: bit 0 = the initiator's live copy W carries steps to apply on top of the
// average, bits 8-15 = the initiator's number of local steps (used when the steps are taken inside the
// interaction kernel).  16 bytes: one scalar load per workgroup.
struct SeqDesc {
    uint32_t ni, nj, event, flags;
};
constexpr uint32_t SEQ_HAS_DELTA = 1u;
// `count` interactions with pairwise disjoint node sets, one grid row each, described by descs_dev
// (device), or the single interaction `one` when descs_dev is null.  local: take the initiators' local
// steps of this diagonal objective in registers (from the snapshot, W untouched), or null.
struct DiagObjective;
hipError_t launch_interact(const GossipArgs &a, uint32_t bits, const SeqDesc *descs_dev, SeqDesc one, uint32_t count,
                           const DiagObjective *local, float lr, hipStream_t st);
hipError_t launch_quantize(const float *x, uint64_t d, float eps, float inv_eps, uint32_t bits,
                           uint64_t seed, uint32_t node, uint32_t event, uint8_t *codes,
                           DeviceCounters *counters, hipStream_t st);
hipError_t launch_dequantize(const uint8_t *codes, const float *key, uint64_t d, float eps, float inv_eps,
                             uint32_t bits, float *out, hipStream_t st);

// Which nodes take local steps in one launch, one entry per grid row ("slot"): device arrays of the
// node id, the number of steps and the event (round or interaction number) that keys the node's
// random streams.  A null array means: node = slot, H steps, the launch's common event.
struct LocalSlots {
    const uint32_t *nodes = nullptr, *steps = nullptr, *events = nullptr;
};

// Local steps, diagonal quadratics, for `count` slots.
hipError_t launch_local_diag(const float *X, float *W, const float *a, const float *c, const LocalSlots &slots,
                             uint32_t count, uint64_t d, uint32_t H, float lr, float sigma, uint64_t seed,
                             uint32_t event, hipStream_t st);

// Round kernels for multi-resolution registers (16-bit code in three planes plus 64-bit tile checksums, read by
// prefixes).  kind: 0 = pairs with any mix of fresh and stale reads, 1 = pairs whose reads are both stale,
// 2 = unmatched nodes (rows = their number).  local: objective of the one-pass round, or null.
hipError_t launch_prefix(const GossipArgs &g, const DiagObjective *local, bool inplace, float lr, int kind, uint32_t rows,
                         hipStream_t st);
// One step of Algorithm 1 with multi-resolution registers: initiator i reads responder j's register.
// `count` interactions with pairwise disjoint node sets (descs_dev, device), or the single one `one`.
hipError_t launch_prefix_interact(const GossipArgs &g, const SeqDesc *descs_dev, SeqDesc one, uint32_t count,
                                  hipStream_t st);
constexpr uint32_t PREFIX_TILE = 512;      // coordinates per checksum (one wave tile)

// One lattice scale per round: state[0] = float bits of the coming round's scale, state[1] = float bits of
// the largest disagreement of the last round that had pairs, state[2 .. 2 + FAR_STRIPES) = the stripes the
// workgroups of the round in flight report their disagreement into (spread so that they do not serialise
// on one address).  Closes a round: m = maximum of the stripes, next scale = max(pair_scale(2 m), eps / 2)
// if the round had pairs, written to the next ring slot's entry of eps_slots; clears the stripes.
constexpr uint32_t FAR_STRIPES = 256;
hipError_t launch_scale_close(float *eps_slots, uint32_t *state, uint32_t slot_now, uint32_t ring_depth,
                              uint32_t bits, uint32_t npairs, hipStream_t st);

// Reductions.  The per-pair distance is the maximum of PAIR_STRIPES words: the workgroups of a pair spread
// their atomic maxima over them (thousands of atomics on one word queue up at its memory channel).
constexpr uint32_t PAIR_STRIPES = 64;
hipError_t launch_potential(const float *X, uint32_t n, uint64_t d, float *mu, double *partials,
                            uint32_t npartials, double *gamma_out, hipStream_t st);
uint32_t potential_partials(uint64_t d);
hipError_t launch_pair_linf(const float *X, uint64_t d, const uint32_t *pairs, uint32_t npairs,
                            uint32_t *linf_bits, hipStream_t st);
// Same reduction over pair descriptors.  For both: linf_bits holds npairs x PAIR_STRIPES words, zero on entry.
hipError_t launch_pair_linf_desc(const float *X, uint64_t d, const PairDesc *pairs, uint32_t npairs,
                                 uint32_t *linf_bits, hipStream_t st);

// Streaming copy of nbytes (multiple of 16, below 2^36) from src to dst.
hipError_t launch_stream_copy(const void *src, void *dst, uint64_t nbytes, hipStream_t st);
// n_read streams of stream_bytes each (consecutive in src) summed into n_write streams (consecutive in
// dst; write stream w gets the sum plus w); supported shapes (n_read, n_write): (2,1), (3,1), (2,2), (4,2), (6,2).
hipError_t launch_stream_mix(const void *src, void *dst, uint64_t stream_bytes, uint32_t n_read, uint32_t n_write,
                             hipStream_t st);

// Matching: one workgroup; outputs pairs (increasing edge index), their count, the
// unmatched nodes and their count.
hipError_t launch_matching(const uint32_t *edges, uint32_t n_edges, uint32_t n, uint64_t seed, uint32_t round,
                           uint32_t *prio_scratch /*n_edges words*/, uint32_t *pairs, uint32_t *singles,
                           uint32_t *counts /*[0]=pairs,[1]=singles*/, hipStream_t st);
constexpr uint32_t MATCHING_MAX_NODES = 4096;
constexpr uint32_t MATCHING_MAX_EDGES = 1u << 20;

}  // namespace swarm
