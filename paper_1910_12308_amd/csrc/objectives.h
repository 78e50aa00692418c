// Node objectives: borrowed data pointers, workspaces and the local-step launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swarm {

struct DiagObjective { const float *a; const float *c; float sigma; };

constexpr uint32_t LSQ_MAX_BATCH = 64;
struct LsqObjective {
    const float *A = nullptr;    // n x m_rows x d
    const float *b = nullptr;    // n x m_rows
    uint32_t m_rows = 0, batch = 0;
    // split form (small swarms): tagged partial residuals exchanged between the workgroups of a node
    // (owned; null when the single-workgroup form is used)
    unsigned long long *part = nullptr;
    size_t part_bytes = 0;
    uint32_t launches = 0;          // launches of the split form so far (24 bits, tags the exchanged words)
};

struct MlpObjective {
    uint32_t n_in = 0, n_hid = 0, n_out = 0, batch = 0;
    const float *means = nullptr;   // n_out x n_in
    const float *cdf = nullptr;     // n x n_out
    float data_sigma = 0.f;
    // workspace for all nodes (owned): inputs, labels, hidden activations, logits gradient, hidden gradient
    float *x = nullptr, *hid = nullptr, *dlogits = nullptr, *dhid = nullptr;
    uint32_t *labels = nullptr;
    uint32_t n_nodes = 0;
    bool bf16x3 = false;            // GEMMs as three bf16 products per term instead of float32 matrix instructions
};

// Whole round in one pass (local steps + quantized gossip) for the diagonal objective; bits in {2,4,8,16}.
struct GossipArgs;
hipError_t launch_fused_pairs(const GossipArgs &g, const DiagObjective &o, uint32_t bits, bool inplace, uint32_t H,
                              float lr, int stale_mode, uint32_t npairs, hipStream_t st);
hipError_t launch_fused_singles(const GossipArgs &g, const DiagObjective &o, uint32_t bits, bool inplace, uint32_t H,
                                float lr, uint32_t nsingles, hipStream_t st);

struct LocalSlots;
struct DeviceCounters;
struct SeqDesc;
// Allocates the exchange buffers of the split form when ceil(d / 512) * n workgroups are few enough to be
// resident together (they wait for one another inside the kernel).
hipError_t alloc_lsq(LsqObjective &o, uint64_t d, uint32_t n);
hipError_t launch_local_lsq(const float *base, float *W, LsqObjective &o, const LocalSlots &slots,
                            DeviceCounters *counters, uint32_t count, uint64_t d, uint32_t H, float lr, uint64_t seed,
                            uint32_t event, hipStream_t st);
// Steps of Algorithm 1 on disjoint nodes in one kernel (split form only): each initiator's local steps
// (count taken from its descriptor) from its snapshot, then its interaction.
hipError_t launch_lsq_interact(const GossipArgs &g, uint32_t bits, const SeqDesc *descs_dev, uint32_t count,
                               LsqObjective &o, float lr, hipStream_t st);
void free_lsq(LsqObjective &o);

hipError_t alloc_mlp(MlpObjective &o, uint32_t n_nodes);
void free_mlp(MlpObjective &o);
hipError_t launch_local_mlp(const float *base, float *W, const MlpObjective &o, const LocalSlots &slots,
                            uint32_t count, uint32_t n, uint64_t d, uint32_t H, float lr, uint64_t seed,
                            uint32_t event, hipStream_t st);

}  // namespace swarm
