// C ABI of the swarm-interaction library: handle, validation, host-side bookkeeping and
// kernel sequencing.  Every arithmetic step of an interaction runs in the kernels of
// this directory; the host code below only validates arguments, keeps the small
// per-round metadata (pairs, unmatched nodes, staleness, pending marks) and enqueues.
#include "swarm.h"
#include "swarm_bench.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "internal.h"
#include "objectives.h"
#include "philox.hpp"

using namespace swarm;

namespace {

constexpr int DESC_SLOTS = 4;   // pinned staging slots for per-round metadata
constexpr uint32_t SEQ_CHUNK = 1u << 15;                              // interactions of Algorithm 1 staged per upload
constexpr size_t SEQ_ENTRY_BYTES = sizeof(swarm::SeqDesc) + 3 * sizeof(uint32_t);

enum ObjectiveKind { OBJ_NONE = 0, OBJ_DIAG, OBJ_LSQ, OBJ_MLP };

}  // namespace

struct swarm_ctx {
    swarm_config cfg{};
    std::vector<uint32_t> edges;                 // 2 per edge, as given
    std::vector<uint64_t> edge_keys;             // sorted (min << 32 | max) for membership tests
    std::vector<std::vector<uint32_t>> adj;      // sorted neighbour lists
    hipStream_t stream = nullptr;
    int device = 0;
    float inv_eps = 0.f;
    uint64_t row_bytes = 0;

    float *X = nullptr, *W = nullptr, *Xhat = nullptr;
    uint8_t *ring = nullptr;
    uint32_t *edges_dev = nullptr, *prio_dev = nullptr, *nodes_dev = nullptr;
    uint32_t *linf_dev = nullptr, *steps_dev = nullptr;   // steps_dev: local steps per slot of a launch (geometric law)
    // batches of Algorithm 1: per interaction a descriptor, the initiator, its step count and its event
    uint8_t *seq_dev = nullptr, *seq_host = nullptr;      // capacity seq_cap interactions each (seq_host pinned)
    uint32_t seq_cap = 0;
    hipEvent_t seq_free = nullptr;                        // the last upload from seq_host has completed
    bool timing_armed = false;                            // HIP events around the passes: off until swarm_timing_reset
    PrefixStats *prefix_stats_dev = nullptr;   // multi-resolution registers: striped escalation counts
    float *eps_slots_dev = nullptr;     // one scale per round: scale of the codes in each ring slot
    uint32_t *scale_state_dev = nullptr; // [0] next scale, [1] disagreement of the last round with pairs, then the stripes
    uint8_t *desc_dev = nullptr;                 // PairDesc[n/2] | singles[n]
    DeviceCounters *counters_dev = nullptr;
    double *partials_dev = nullptr, *gamma_dev = nullptr;

    // pinned host staging
    uint8_t *desc_host[DESC_SLOTS] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t desc_free[DESC_SLOTS] = {nullptr, nullptr, nullptr, nullptr};
    unsigned desc_next = 0;
    uint32_t *match_host = nullptr;              // counts[2] | pairs | singles
    uint32_t *match_dev = nullptr;               // match_host as the device sees it: the matching kernel writes there
    hipStream_t match_stream = nullptr;          // the matching runs beside the round kernels, not between them
    hipEvent_t match_ready = nullptr;            // the matching of round match_round has reached match_host
    uint64_t match_round = ~0ull;
    double *scalar_host = nullptr;

    size_t off_pairs = 0, off_singles = 0, desc_bytes = 0;

    std::vector<uint8_t> pending;                // host mirror: W_i carries unapplied steps
    ObjectiveKind kind = OBJ_NONE;
    DiagObjective diag{};
    LsqObjective lsq{};
    MlpObjective mlp{};

    uint64_t round = 0, interactions = 0, bits_communicated = 0;
    uint64_t prefix_tile_reads = 0;      // multi-resolution registers: tiles read since init
    std::vector<hipEvent_t> ev_gossip, ev_local;   // start/stop pairs, created on demand
    uint32_t timed_gossip = 0, timed_local = 0;    // recorded calls since the last reset
    std::string err;

    PairDesc *pairs_dev() const { return (PairDesc *)(desc_dev + off_pairs); }
    uint32_t *singles_dev() const { return (uint32_t *)(desc_dev + off_singles); }
};

namespace {

thread_local std::string g_init_error;

}  // namespace

void swarm::set_global_error(const char *message) { g_init_error = message; }

namespace {

swarm_status fail(swarm_t h, swarm_status code, const std::string &msg) {
    if (h) h->err = msg; else g_init_error = msg;
    return code;
}

#define SWARM_HIP(h, expr)                                                                          \
    do {                                                                                            \
        hipError_t e_ = (expr);                                                                     \
        if (e_ != hipSuccess)                                                                       \
            return fail(h, e_ == hipErrorOutOfMemory ? SWARM_ENOMEM : SWARM_EDEVICE,                \
                        std::string(#expr) + ": " + hipGetErrorString(e_));                         \
    } while (0)

bool valid_bits(uint32_t b) { return b == 2 || b == 4 || b == 8 || b == 16; }

uint64_t edge_key(uint32_t u, uint32_t v) { return ((uint64_t)std::min(u, v) << 32) | std::max(u, v); }

GossipArgs gossip_args(swarm_t h, uint32_t event, uint32_t slot) {
    GossipArgs a{};
    a.X = h->X; a.W = h->W; a.Xhat = h->Xhat; a.ring = h->ring;
    a.pairs = h->pairs_dev(); a.singles = h->singles_dev();
    a.counters = h->counters_dev;
    a.d = h->cfg.d; a.row_bytes = h->row_bytes; a.seed = h->cfg.seed;
    a.n = h->cfg.n; a.event = event; a.slot_now = slot; a.ring_depth = h->cfg.stale_max + 1;
    a.eps = h->cfg.eps; a.inv_eps = h->inv_eps;
    a.eps_slots = h->eps_slots_dev;
    a.prefix_stats = h->prefix_stats_dev;
    a.far_bits = h->scale_state_dev ? h->scale_state_dev + 2 : nullptr;
    return a;
}

// Take the next pinned staging slot once the copy that last used it has completed.
swarm_status acquire_desc(swarm_t h, uint8_t **slot, unsigned *index) {
    const unsigned s = h->desc_next++ % DESC_SLOTS;
    SWARM_HIP(h, hipEventSynchronize(h->desc_free[s]));
    *slot = h->desc_host[s];
    *index = s;
    return SWARM_OK;
}

// Snapshots (models at the last initiation) start equal to the current models.
swarm_status ensure_snapshots(swarm_t h) {
    if (h->Xhat) return SWARM_OK;
    const size_t model_bytes = (size_t)h->cfg.n * h->cfg.d * sizeof(float);
    SWARM_HIP(h, hipMalloc((void **)&h->Xhat, model_bytes));
    SWARM_HIP(h, hipMemcpyAsync(h->Xhat, h->X, model_bytes, hipMemcpyDeviceToDevice, h->stream));
    return SWARM_OK;
}

static_assert(MATCHING_MAX_NODES <= SINGLE_NODE_MASK, "node ids must fit the unmatched-node entries");
constexpr uint32_t MAX_TIMED_CALLS = 1024;

// Record the start (which = 0) or stop (which = 1) event of timed call number `call`.
swarm_status record_timing(swarm_t h, std::vector<hipEvent_t> &events, uint32_t call, int which) {
    if (!h->timing_armed || call >= MAX_TIMED_CALLS) return SWARM_OK;
    while (events.size() < 2 * (size_t)(call + 1)) {
        hipEvent_t e = nullptr;
        SWARM_HIP(h, hipEventCreate(&e));
        events.push_back(e);
    }
    SWARM_HIP(h, hipEventRecord(events[2 * call + which], h->stream));
    return SWARM_OK;
}

#define SWARM_TRY(expr)                     \
    do {                                    \
        const swarm_status rc_ = (expr);    \
        if (rc_ != SWARM_OK) return rc_;    \
    } while (0)

// Stage a small host array of node ids in pinned memory and copy it to nodes_dev on the stream
// (the caller's array may be reused as soon as the call returns).
swarm_status upload_nodes(swarm_t h, const uint32_t *ids, uint32_t count) {
    uint8_t *slot = nullptr;
    unsigned slot_index = 0;
    SWARM_TRY(acquire_desc(h, &slot, &slot_index));
    std::memcpy(slot, ids, sizeof(uint32_t) * count);
    SWARM_HIP(h, hipMemcpyAsync(h->nodes_dev, slot, sizeof(uint32_t) * count, hipMemcpyHostToDevice, h->stream));
    SWARM_HIP(h, hipEventRecord(h->desc_free[slot_index], h->stream));
    return SWARM_OK;
}

// Number of local steps of `node` for interaction `event`: H, or a geometric draw of mean H
// (1 + failures before the first word below floor(2^32 / H), words taken in order from the
// node's STEPS stream), capped at 255.
uint32_t draw_steps(const swarm_config &c, uint32_t node, uint32_t event) {
    if (c.steps_law == SWARM_STEPS_CONSTANT) return c.H;
    const uint32_t threshold = (uint32_t)((1ull << 32) / c.H);   // H = 1 -> 2^32 wraps to 0: handled below
    if (c.H == 1) return 1;
    uint32_t k = 1;
    for (uint32_t call = 0; k < 255; ++call) {
        const Words4 w = stream(c.seed, TAG_STEPS, 0, node, event, call);
        const uint32_t words[4] = {w.w0, w.w1, w.w2, w.w3};
        for (int t = 0; t < 4 && k < 255; ++t) {
            if (words[t] < threshold) return k;
            ++k;
        }
    }
    return k;
}

// Step counts of this event on the device, one word per slot of the launch (slot k = node ids[k], or
// node k when ids is null), or null when the number of steps is constant.
swarm_status upload_steps(swarm_t h, uint32_t event, const uint32_t *ids, uint32_t count, const uint32_t **steps_dev) {
    *steps_dev = nullptr;
    if (h->cfg.steps_law == SWARM_STEPS_CONSTANT) return SWARM_OK;
    uint8_t *slot = nullptr;
    unsigned slot_index = 0;
    SWARM_TRY(acquire_desc(h, &slot, &slot_index));
    uint32_t *dst = (uint32_t *)slot;
    for (uint32_t k = 0; k < count; ++k) dst[k] = draw_steps(h->cfg, ids ? ids[k] : k, event);
    SWARM_HIP(h, hipMemcpyAsync(h->steps_dev, slot, sizeof(uint32_t) * count, hipMemcpyHostToDevice, h->stream));
    SWARM_HIP(h, hipEventRecord(h->desc_free[slot_index], h->stream));
    *steps_dev = h->steps_dev;
    return SWARM_OK;
}

// Enqueue the local-step kernels of the objective for `count` slots.
swarm_status launch_local(swarm_t h, const float *base, const LocalSlots &slots, uint32_t count, uint32_t event) {
    const swarm_config &c = h->cfg;
    hipError_t e = hipSuccess;
    switch (h->kind) {
        case OBJ_DIAG:
            e = launch_local_diag(base, h->W, h->diag.a, h->diag.c, slots, count, c.d, c.H, c.lr, h->diag.sigma, c.seed,
                                  event, h->stream);
            break;
        case OBJ_LSQ:
            e = launch_local_lsq(base, h->W, h->lsq, slots, h->counters_dev, count, c.d, c.H, c.lr, c.seed, event, h->stream);
            break;
        case OBJ_MLP:
            e = launch_local_mlp(base, h->W, h->mlp, slots, count, c.n, c.d, c.H, c.lr, c.seed, event, h->stream);
            break;
        default:
            return fail(h, SWARM_ESTATE, "no objective set");
    }
    SWARM_HIP(h, e);
    return SWARM_OK;
}

// ids: host list of the nodes in nodes_dev (already uploaded), or null for all nodes.
swarm_status run_local_steps(swarm_t h, const float *base, const uint32_t *ids, const uint32_t *nodes_dev, uint32_t count,
                             uint32_t event) {
    if (h->kind == OBJ_MLP && h->cfg.steps_law != SWARM_STEPS_CONSTANT)
        return fail(h, SWARM_ESTATE, "the MLP objective takes a constant number of local steps");
    LocalSlots slots;
    slots.nodes = nodes_dev;
    SWARM_TRY(upload_steps(h, event, ids, count, &slots.steps));
    return launch_local(h, base, slots, count, event);
}

}  // namespace

extern "C" {

const char *swarm_last_error(swarm_t h) { return h ? h->err.c_str() : g_init_error.c_str(); }

swarm_status swarm_init(const swarm_config *cfg, const float *x0_dev, void *hip_stream, swarm_t *out) {
    if (!cfg || !out) return fail(nullptr, SWARM_EINVAL, "null config or output");
    *out = nullptr;
    if (cfg->n < 2) return fail(nullptr, SWARM_EINVAL, "n must be >= 2");
    if (cfg->n > MATCHING_MAX_NODES) return fail(nullptr, SWARM_EINVAL, "n exceeds 4096");
    if (cfg->d == 0 || cfg->d % 8 != 0) return fail(nullptr, SWARM_EINVAL, "d must be a positive multiple of 8");
    if (cfg->bits != 0 && !valid_bits(cfg->bits)) return fail(nullptr, SWARM_EINVAL, "bits must be 0, 2, 4, 8 or 16");
    if (cfg->bits != 0 && !(cfg->eps > 0.f) ) return fail(nullptr, SWARM_EINVAL, "eps must be positive");
    if (cfg->bits == 0 && cfg->stale_max != 0) return fail(nullptr, SWARM_EINVAL, "stale reads need quantized codes");
    if (cfg->stale_max > 254) return fail(nullptr, SWARM_EINVAL, "stale_max exceeds 254");
    if (cfg->H > 255) return fail(nullptr, SWARM_EINVAL, "H exceeds 255");
    if (cfg->apply_mode > SWARM_APPLY_INPLACE) return fail(nullptr, SWARM_EINVAL, "unknown apply mode");
    if (cfg->steps_law > SWARM_STEPS_GEOMETRIC) return fail(nullptr, SWARM_EINVAL, "unknown law of the local steps");
    if (cfg->steps_law == SWARM_STEPS_GEOMETRIC && cfg->H == 0)
        return fail(nullptr, SWARM_EINVAL, "a geometric number of local steps needs mean H >= 1");
    if (cfg->scale_policy > SWARM_SCALE_GLOBAL_LINF) return fail(nullptr, SWARM_EINVAL, "unknown scale policy");
    if (cfg->scale_policy == SWARM_SCALE_GLOBAL_LINF) {
        int exponent;
        if (cfg->bits < 8 || std::frexp(cfg->eps, &exponent) != 0.5f)
            return fail(nullptr, SWARM_EINVAL, "the per-round scale needs bits >= 8 and a power of two as starting eps");
    }
    if (cfg->scale_policy == SWARM_SCALE_PAIR_LINF && (cfg->bits < 4 || cfg->stale_max != 0))
        return fail(nullptr, SWARM_EINVAL, "the per-pair scale needs bits >= 4 and stale_max = 0");
    if (cfg->codec > SWARM_CODEC_PREFIX) return fail(nullptr, SWARM_EINVAL, "unknown codec");
    if (cfg->codec == SWARM_CODEC_PREFIX && (cfg->bits != 16 || cfg->scale_policy != SWARM_SCALE_FIXED))
        return fail(nullptr, SWARM_EINVAL, "multi-resolution registers need bits = 16 and the fixed lattice scale");
    if (cfg->n_edges == 0 || !cfg->edges) return fail(nullptr, SWARM_EINVAL, "graph has no edges");
    if (cfg->n_edges > MATCHING_MAX_EDGES) return fail(nullptr, SWARM_EINVAL, "too many edges");

    swarm_ctx *h = new (std::nothrow) swarm_ctx();
    if (!h) return fail(nullptr, SWARM_ENOMEM, "host allocation failed");
    h->cfg = *cfg;
    h->edges.assign(cfg->edges, cfg->edges + 2 * (size_t)cfg->n_edges);
    h->cfg.edges = h->edges.data();
    h->adj.resize(cfg->n);
    for (uint32_t e = 0; e < cfg->n_edges; ++e) {
        const uint32_t u = h->edges[2 * e], v = h->edges[2 * e + 1];
        if (u >= cfg->n || v >= cfg->n || u == v) {
            delete h;
            return fail(nullptr, SWARM_EINVAL, "edge endpoint out of range or self loop");
        }
        h->edge_keys.push_back(edge_key(u, v));
        h->adj[u].push_back(v);
        h->adj[v].push_back(u);
    }
    std::sort(h->edge_keys.begin(), h->edge_keys.end());
    if (std::adjacent_find(h->edge_keys.begin(), h->edge_keys.end()) != h->edge_keys.end()) {
        delete h;
        return fail(nullptr, SWARM_EINVAL, "duplicate edge");
    }
    for (auto &a : h->adj) std::sort(a.begin(), a.end());
    h->stream = (hipStream_t)hip_stream;
    h->inv_eps = cfg->bits ? 1.0f / cfg->eps : 0.f;
    h->row_bytes = cfg->d * cfg->bits / 8;
    if (cfg->codec == SWARM_CODEC_PREFIX)            // three planes (2 d bytes) and one 64-bit checksum per tile
        h->row_bytes += 2 * sizeof(uint32_t) * ((cfg->d + PREFIX_TILE - 1) / PREFIX_TILE);
    h->pending.assign(cfg->n, 0);

    const uint32_t n = cfg->n;
    h->off_pairs = 0;
    h->off_singles = h->off_pairs + sizeof(PairDesc) * (n / 2);
    h->desc_bytes = h->off_singles + sizeof(uint32_t) * n;

    swarm_status rc = SWARM_OK;
    auto body = [&]() -> swarm_status {
        SWARM_HIP(h, hipGetDevice(&h->device));
        const size_t model_bytes = (size_t)n * cfg->d * sizeof(float);
        SWARM_HIP(h, hipMalloc((void **)&h->X, model_bytes));
        if (cfg->apply_mode == SWARM_APPLY_INPLACE) h->W = h->X;     // one matrix: local steps update X itself
        else SWARM_HIP(h, hipMalloc((void **)&h->W, model_bytes));
        if (cfg->bits) {
            const size_t ring_bytes = (size_t)(cfg->stale_max + 1) * n * h->row_bytes;
            SWARM_HIP(h, hipMalloc((void **)&h->ring, ring_bytes));
            SWARM_HIP(h, hipMemsetAsync(h->ring, 0, ring_bytes, h->stream));   // registers start as zero vectors
        }
        SWARM_HIP(h, hipMalloc((void **)&h->edges_dev, sizeof(uint32_t) * 2 * cfg->n_edges));
        SWARM_HIP(h, hipMalloc((void **)&h->prio_dev, sizeof(uint32_t) * cfg->n_edges));
        SWARM_HIP(h, hipMalloc((void **)&h->nodes_dev, sizeof(uint32_t) * n));
        SWARM_HIP(h, hipMalloc((void **)&h->linf_dev, sizeof(uint32_t) * PAIR_STRIPES * (n / 2)));
        SWARM_HIP(h, hipMalloc((void **)&h->steps_dev, sizeof(uint32_t) * n));
        if (cfg->codec == SWARM_CODEC_PREFIX) {
            SWARM_HIP(h, hipMalloc((void **)&h->prefix_stats_dev, sizeof(PrefixStats) * PREFIX_STRIPES));
            SWARM_HIP(h, hipMemsetAsync(h->prefix_stats_dev, 0, sizeof(PrefixStats) * PREFIX_STRIPES, h->stream));
        }
        if (cfg->scale_policy == SWARM_SCALE_GLOBAL_LINF) {
            const std::vector<float> slots(cfg->stale_max + 1, cfg->eps);
            std::vector<uint32_t> state(2 + FAR_STRIPES, 0u);
            std::memcpy(&state[0], &cfg->eps, sizeof(float));
            SWARM_HIP(h, hipMalloc((void **)&h->eps_slots_dev, sizeof(float) * slots.size()));
            SWARM_HIP(h, hipMalloc((void **)&h->scale_state_dev, sizeof(uint32_t) * state.size()));
            SWARM_HIP(h, hipMemcpy(h->eps_slots_dev, slots.data(), sizeof(float) * slots.size(), hipMemcpyHostToDevice));
            SWARM_HIP(h, hipMemcpy(h->scale_state_dev, state.data(), sizeof(uint32_t) * state.size(), hipMemcpyHostToDevice));
        }
        SWARM_HIP(h, hipMalloc((void **)&h->desc_dev, h->desc_bytes));
        SWARM_HIP(h, hipEventCreateWithFlags(&h->match_ready, hipEventDisableTiming));
        SWARM_HIP(h, hipMalloc((void **)&h->counters_dev, sizeof(DeviceCounters)));
        SWARM_HIP(h, hipMalloc((void **)&h->partials_dev, sizeof(double) * potential_partials(cfg->d)));
        SWARM_HIP(h, hipMalloc((void **)&h->gamma_dev, sizeof(double)));
        for (int s = 0; s < DESC_SLOTS; ++s) {
            SWARM_HIP(h, hipHostMalloc((void **)&h->desc_host[s], h->desc_bytes, hipHostMallocDefault));
            SWARM_HIP(h, hipEventCreateWithFlags(&h->desc_free[s], hipEventDisableTiming));
            SWARM_HIP(h, hipEventRecord(h->desc_free[s], h->stream));
        }
        SWARM_HIP(h, hipHostMalloc((void **)&h->match_host, sizeof(uint32_t) * (2 + 2 * (n / 2) + n),
                                   hipHostMallocDefault));
        SWARM_HIP(h, hipHostGetDevicePointer((void **)&h->match_dev, h->match_host, 0));
        SWARM_HIP(h, hipStreamCreateWithFlags(&h->match_stream, hipStreamNonBlocking));
        SWARM_HIP(h, hipHostMalloc((void **)&h->scalar_host, 64, hipHostMallocDefault));
        SWARM_HIP(h, hipMemcpyAsync(h->edges_dev, h->edges.data(), sizeof(uint32_t) * 2 * cfg->n_edges,
                                    hipMemcpyHostToDevice, h->stream));
        SWARM_HIP(h, hipMemsetAsync(h->counters_dev, 0, sizeof(DeviceCounters), h->stream));
        SWARM_HIP(h, hipMemsetAsync(h->desc_dev, 0, h->desc_bytes, h->stream));
        if (x0_dev) {
            for (uint32_t i = 0; i < n; ++i)     // every node starts from the same model
                SWARM_HIP(h, hipMemcpyAsync(h->X + (uint64_t)i * cfg->d, x0_dev, cfg->d * sizeof(float),
                                            hipMemcpyDeviceToDevice, h->stream));
        } else {
            SWARM_HIP(h, hipMemsetAsync(h->X, 0, model_bytes, h->stream));
        }
        if (h->W != h->X)
            SWARM_HIP(h, hipMemcpyAsync(h->W, h->X, model_bytes, hipMemcpyDeviceToDevice, h->stream));
        SWARM_HIP(h, hipStreamSynchronize(h->stream));
        return SWARM_OK;
    };
    rc = body();
    if (rc != SWARM_OK) {
        g_init_error = h->err;
        swarm_destroy(h);
        return rc;
    }
    *out = h;
    return SWARM_OK;
}

swarm_status swarm_destroy(swarm_t h) {
    if (!h) return SWARM_OK;
    (void)hipStreamSynchronize(h->stream);
    free_lsq(h->lsq);
    free_mlp(h->mlp);
    if (h->W == h->X) h->W = nullptr;
    if (h->match_stream) {
        (void)hipStreamSynchronize(h->match_stream);
        (void)hipStreamDestroy(h->match_stream);
    }
    void *dev[] = {h->X, h->W, h->Xhat, h->ring, h->edges_dev, h->prio_dev, h->nodes_dev,
                   h->linf_dev, h->desc_dev, h->counters_dev, h->partials_dev, h->gamma_dev,
                   h->steps_dev, h->eps_slots_dev, h->scale_state_dev, h->prefix_stats_dev};
    for (void *p : dev) if (p) (void)hipFree(p);
    for (int s = 0; s < DESC_SLOTS; ++s) {
        if (h->desc_host[s]) (void)hipHostFree(h->desc_host[s]);
        if (h->desc_free[s]) (void)hipEventDestroy(h->desc_free[s]);
    }
    if (h->match_host) (void)hipHostFree(h->match_host);
    if (h->match_ready) (void)hipEventDestroy(h->match_ready);
    if (h->scalar_host) (void)hipHostFree(h->scalar_host);
    if (h->seq_dev) (void)hipFree(h->seq_dev);
    if (h->seq_host) (void)hipHostFree(h->seq_host);
    if (h->seq_free) (void)hipEventDestroy(h->seq_free);
    for (hipEvent_t e : h->ev_gossip) (void)hipEventDestroy(e);
    for (hipEvent_t e : h->ev_local) (void)hipEventDestroy(e);
    delete h;
    return SWARM_OK;
}

swarm_status swarm_set_objective_diag(swarm_t h, const float *a_dev, const float *c_dev, float sigma) {
    if (!h) return SWARM_EINVAL;
    if (!a_dev || !c_dev || !(sigma >= 0.f)) return fail(h, SWARM_EINVAL, "diag objective: null data or negative sigma");
    h->diag = DiagObjective{a_dev, c_dev, sigma};
    h->kind = OBJ_DIAG;
    return SWARM_OK;
}

swarm_status swarm_set_objective_lsq(swarm_t h, const float *A_dev, const float *b_dev, uint32_t m_rows,
                                     uint32_t batch) {
    if (!h) return SWARM_EINVAL;
    if (!A_dev || !b_dev || m_rows == 0 || batch == 0 || batch % 4 != 0 || batch > LSQ_MAX_BATCH)
        return fail(h, SWARM_EINVAL, "lsq objective: batch must be a multiple of 4, at most 64");
    free_lsq(h->lsq);
    h->lsq = LsqObjective{};
    h->lsq.A = A_dev; h->lsq.b = b_dev; h->lsq.m_rows = m_rows; h->lsq.batch = batch;
    const hipError_t e = alloc_lsq(h->lsq, h->cfg.d, h->cfg.n);
    if (e != hipSuccess) return fail(h, e == hipErrorOutOfMemory ? SWARM_ENOMEM : SWARM_EDEVICE,
                                     std::string("least-squares exchange buffers: ") + hipGetErrorString(e));
    h->kind = OBJ_LSQ;
    return SWARM_OK;
}

swarm_status swarm_set_objective_mlp(swarm_t h, uint32_t n_in, uint32_t n_hid, uint32_t n_out,
                                     const float *class_means_dev, const float *label_cdf_dev, float data_sigma,
                                     uint32_t batch) {
    if (!h) return SWARM_EINVAL;
    if (!class_means_dev || !label_cdf_dev) return fail(h, SWARM_EINVAL, "mlp objective: null data");
    if (n_in % 32 || n_hid % 32 || n_out % 32 || batch % 32 || !n_in || !n_hid || !n_out || !batch)
        return fail(h, SWARM_EINVAL, "mlp objective: sizes must be positive multiples of 32");
    if ((uint64_t)n_hid * n_in + n_hid + (uint64_t)n_out * n_hid + n_out != h->cfg.d)
        return fail(h, SWARM_EINVAL, "mlp objective: d != hid*in + hid + out*hid + out");
    free_mlp(h->mlp);
    h->mlp = MlpObjective{};
    h->mlp.n_in = n_in; h->mlp.n_hid = n_hid; h->mlp.n_out = n_out; h->mlp.batch = batch;
    h->mlp.means = class_means_dev; h->mlp.cdf = label_cdf_dev; h->mlp.data_sigma = data_sigma;
    const hipError_t e = alloc_mlp(h->mlp, h->cfg.n);
    if (e != hipSuccess) return fail(h, e == hipErrorOutOfMemory ? SWARM_ENOMEM : SWARM_EDEVICE,
                                     std::string("mlp workspace: ") + hipGetErrorString(e));
    h->kind = OBJ_MLP;
    return SWARM_OK;
}

swarm_status swarm_set_mlp_arithmetic(swarm_t h, uint32_t arithmetic) {
    if (!h) return SWARM_EINVAL;
    if (h->kind != OBJ_MLP) return fail(h, SWARM_ESTATE, "the MLP objective is not set");
    if (arithmetic > SWARM_MLP_BF16X3) return fail(h, SWARM_EINVAL, "unknown MLP arithmetic");
    h->mlp.bf16x3 = arithmetic == SWARM_MLP_BF16X3;
    return SWARM_OK;
}

swarm_status swarm_local_steps(swarm_t h, const uint32_t *nodes, uint32_t count) {
    if (!h) return SWARM_EINVAL;
    if (h->kind == OBJ_NONE) return fail(h, SWARM_ESTATE, "no objective set");
    if (h->cfg.H == 0) return SWARM_OK;          // no steps: nothing becomes pending
    const uint32_t n = h->cfg.n;
    const uint32_t *nodes_dev = nullptr;
    if (nodes) {
        if (count == 0 || count > n) return fail(h, SWARM_EINVAL, "node count out of range");
        std::vector<uint8_t> seen(n, 0);
        for (uint32_t k = 0; k < count; ++k) {
            if (nodes[k] >= n || seen[nodes[k]]) return fail(h, SWARM_EINVAL, "node id out of range or repeated");
            seen[nodes[k]] = 1;
        }
        SWARM_TRY(upload_nodes(h, nodes, count));
        nodes_dev = h->nodes_dev;
    } else {
        count = n;
    }
    SWARM_TRY(record_timing(h, h->ev_local, h->timed_local, 0));
    SWARM_TRY(run_local_steps(h, h->X, nodes, nodes_dev, count, (uint32_t)h->round));
    SWARM_TRY(record_timing(h, h->ev_local, h->timed_local, 1));
    h->timed_local += 1;
    if (h->cfg.apply_mode == SWARM_APPLY_INPLACE) return SWARM_OK;   // already applied: nothing is pending
    if (nodes) for (uint32_t k = 0; k < count; ++k) h->pending[nodes[k]] = 1;
    else std::fill(h->pending.begin(), h->pending.end(), 1);
    return SWARM_OK;
}

swarm_status swarm_mark_pending(swarm_t h, const uint32_t *nodes, uint32_t count) {
    if (!h) return SWARM_EINVAL;
    if (h->cfg.apply_mode == SWARM_APPLY_INPLACE)
        return fail(h, SWARM_ESTATE, "in-place apply: update the exchanged models directly, nothing is pending");
    const uint32_t n = h->cfg.n;
    if (!nodes) {
        std::fill(h->pending.begin(), h->pending.end(), 1);
        return SWARM_OK;
    }
    if (count == 0 || count > n) return fail(h, SWARM_EINVAL, "node count out of range");
    std::vector<uint8_t> seen(n, 0);
    for (uint32_t k = 0; k < count; ++k) {
        if (nodes[k] >= n || seen[nodes[k]]) return fail(h, SWARM_EINVAL, "node id out of range or repeated");
        seen[nodes[k]] = 1;
    }
    for (uint32_t k = 0; k < count; ++k) h->pending[nodes[k]] = 1;
    return SWARM_OK;
}

// Enqueue the matching of a round.  It depends only on (seed, round, graph), so it is issued a round
// ahead, on a stream of its own (it runs beside the round kernels instead of between them), and it
// writes its few hundred bytes of results (counts | pairs | unmatched nodes) straight into pinned host
// memory: the host finds them ready instead of draining the stream, and no copy is launched.
static swarm_status enqueue_matching(swarm_t h, uint64_t round) {
    const swarm_config &c = h->cfg;
    const uint32_t maxp = c.n / 2;
    SWARM_HIP(h, launch_matching(h->edges_dev, c.n_edges, c.n, c.seed, (uint32_t)round, h->prio_dev,
                                 h->match_dev + 2, h->match_dev + 2 + 2 * maxp, h->match_dev, h->match_stream));
    SWARM_HIP(h, hipEventRecord(h->match_ready, h->match_stream));
    h->match_round = round;
    return SWARM_OK;
}

static swarm_status sample_matching_device(swarm_t h, uint32_t *npairs, uint32_t *nsingles) {
    const swarm_config &c = h->cfg;
    if (h->match_round != h->round) SWARM_TRY(enqueue_matching(h, h->round));
    SWARM_HIP(h, hipEventSynchronize(h->match_ready));
    *npairs = h->match_host[0];
    *nsingles = h->match_host[1];
    if (*npairs > c.n / 2 || *nsingles > c.n || 2 * *npairs + *nsingles != c.n)
        return fail(h, SWARM_EDEVICE, "matching kernel returned inconsistent counts");
    return SWARM_OK;
}

swarm_status swarm_sample_matching(swarm_t h, uint32_t *pairs_host, uint32_t *npairs) {
    if (!h) return SWARM_EINVAL;
    if (!pairs_host || !npairs) return fail(h, SWARM_EINVAL, "null output");
    uint32_t np = 0, ns = 0;
    const swarm_status rc = sample_matching_device(h, &np, &ns);
    if (rc != SWARM_OK) return rc;
    std::memcpy(pairs_host, h->match_host + 2, sizeof(uint32_t) * 2 * np);
    *npairs = np;
    return SWARM_OK;
}

swarm_status swarm_sample_stale(swarm_t h, uint8_t *stale_host) {
    if (!h) return SWARM_EINVAL;
    if (!stale_host) return fail(h, SWARM_EINVAL, "null output");
    for (uint32_t i = 0; i < h->cfg.n; ++i) {
        const uint32_t s = scaled_index(stream(h->cfg.seed, TAG_STALE, 0, i, (uint32_t)h->round, 0).w0,
                                        h->cfg.stale_max + 1);
        stale_host[i] = (uint8_t)std::min<uint64_t>(s, h->round);
    }
    return SWARM_OK;
}

swarm_status swarm_sample_steps(swarm_t h, uint8_t *steps_host) {
    if (!h) return SWARM_EINVAL;
    if (!steps_host) return fail(h, SWARM_EINVAL, "null output");
    for (uint32_t i = 0; i < h->cfg.n; ++i) steps_host[i] = (uint8_t)draw_steps(h->cfg, i, (uint32_t)h->round);
    return SWARM_OK;
}

swarm_status swarm_sample_pair(swarm_t h, uint32_t *i, uint32_t *j) {
    if (!h) return SWARM_EINVAL;
    if (!i || !j) return fail(h, SWARM_EINVAL, "null output");
    const Words4 w = stream(h->cfg.seed, TAG_PICK, 0, 0, (uint32_t)h->interactions, 0);
    *i = scaled_index(w.w0, h->cfg.n);
    const std::vector<uint32_t> &nb = h->adj[*i];
    if (nb.empty()) return fail(h, SWARM_ESTATE, "initiator has no neighbour");
    *j = nb[scaled_index(w.w1, (uint32_t)nb.size())];
    return SWARM_OK;
}

static swarm_status round_impl(swarm_t h, const uint32_t *pairs_host, uint32_t npairs, const uint8_t *stale_host,
                               bool fused) {
    const swarm_config &c = h->cfg;
    const bool pair_scale_policy = c.scale_policy == SWARM_SCALE_PAIR_LINF;
    if (fused) {
        if (pair_scale_policy) return fail(h, SWARM_ESTATE, "the one-pass round cannot use the per-pair lattice scale");
        if (h->kind != OBJ_DIAG) return fail(h, SWARM_ESTATE, "the fused round needs the diagonal-quadratic objective");
        if (c.bits == 0 || c.H == 0) return fail(h, SWARM_ESTATE, "the fused round needs quantized codes and H > 0");
        for (uint8_t p : h->pending)
            if (p) return fail(h, SWARM_ESTATE, "local steps are already pending: use swarm_gossip_round");
    }
    const uint32_t n = c.n;
    std::vector<uint32_t> pairs, singles;
    uint32_t nsingles = 0;
    if (pairs_host) {
        if (npairs > n / 2) return fail(h, SWARM_EINVAL, "more pairs than floor(n/2)");
        std::vector<uint8_t> used(n, 0);
        for (uint32_t p = 0; p < npairs; ++p) {
            const uint32_t u = pairs_host[2 * p], v = pairs_host[2 * p + 1];
            if (u >= n || v >= n || u == v) return fail(h, SWARM_EINVAL, "pair endpoint out of range");
            if (!std::binary_search(h->edge_keys.begin(), h->edge_keys.end(), edge_key(u, v)))
                return fail(h, SWARM_EINVAL, "pair is not an edge of the graph");
            if (used[u] || used[v]) return fail(h, SWARM_EINVAL, "node appears in two pairs");
            used[u] = used[v] = 1;
        }
        pairs.assign(pairs_host, pairs_host + 2 * (size_t)npairs);
        for (uint32_t u = 0; u < n; ++u) if (!used[u]) singles.push_back(u);
        nsingles = (uint32_t)singles.size();
    } else {
        const swarm_status rc = sample_matching_device(h, &npairs, &nsingles);
        if (rc != SWARM_OK) return rc;
        pairs.assign(h->match_host + 2, h->match_host + 2 + 2 * (size_t)npairs);
        singles.assign(h->match_host + 2 + 2 * (n / 2), h->match_host + 2 + 2 * (n / 2) + nsingles);
        // The next round's matching goes into the stream now, ahead of this round's long kernels, so
        // that the next call finds it ready without waiting for them (match_host was copied out above).
        SWARM_TRY(enqueue_matching(h, h->round + 1));
    }
    std::vector<uint8_t> stale(n, 0);
    if (stale_host) {
        for (uint32_t u = 0; u < n; ++u) {
            if (stale_host[u] > c.stale_max) return fail(h, SWARM_EINVAL, "staleness exceeds stale_max");
            stale[u] = (uint8_t)std::min<uint64_t>(stale_host[u], h->round);   // only rounds that exist
        }
    }
    // Which kernel specialisations serve the pairs?  Pending marks: all / none / mixed.  Staleness:
    // pairs are grouped into both-fresh, both-stale and one-stale (stale reader listed first), and
    // each group gets the kernel compiled for it; with mixed pending marks one generic launch is used.
    uint32_t with_delta = 0;
    for (uint32_t k = 0; k < 2 * npairs; ++k) with_delta += h->pending[pairs[k]] != 0;
    const int delta_mode = with_delta == 0 ? 0 : (with_delta == 2 * npairs ? 1 : 2);
    std::vector<PairDesc> groups[3];          // 0: fresh/fresh, 1: stale/stale, 2: first stale only
    auto describe = [&](uint32_t u, uint32_t v) {
        return PairDesc{u, v, (uint32_t)stale[u] | ((uint32_t)stale[v] << 8) |
                                  (h->pending[u] ? 1u << 16 : 0u) | (h->pending[v] ? 1u << 17 : 0u),
                        fused ? draw_steps(c, u, (uint32_t)h->round) | (draw_steps(c, v, (uint32_t)h->round) << 8) : 0u};
    };
    for (uint32_t p = 0; p < npairs; ++p) {
        const uint32_t u = pairs[2 * p], v = pairs[2 * p + 1];
        if (delta_mode == 2) groups[0].push_back(describe(u, v));
        else if (!stale[u] && !stale[v]) groups[0].push_back(describe(u, v));
        else if (stale[u] && stale[v]) groups[1].push_back(describe(u, v));
        else if (stale[u]) groups[2].push_back(describe(u, v));
        else groups[2].push_back(describe(v, u));
    }
    const int group_mode[3] = {delta_mode == 2 ? 2 : 0, 1, 3};

    // Per-round metadata: one descriptor per pair (nodes, staleness, pending flags) and the unmatched
    // nodes, staged in pinned memory and copied with one transfer.  (Carrying them in the kernel arguments
    // of small rounds instead was measured: the copy costs the step nothing, a second source of descriptors
    // costs the kernels 0.5 to 2 %.)
    {
        uint8_t *slot = nullptr;
        unsigned slot_index = 0;
        const swarm_status rc = acquire_desc(h, &slot, &slot_index);
        if (rc != SWARM_OK) return rc;
        PairDesc *pd = (PairDesc *)(slot + h->off_pairs);
        for (int gidx = 0; gidx < 3; ++gidx)
            for (const PairDesc &desc : groups[gidx]) *pd++ = desc;
        uint32_t *sg = (uint32_t *)(slot + h->off_singles);
        for (uint32_t k = 0; k < nsingles; ++k)
            sg[k] = singles[k] | (fused ? draw_steps(c, singles[k], (uint32_t)h->round) << 16 : 0u) |
                    (h->pending[singles[k]] ? SINGLE_PENDING : 0u);
        SWARM_HIP(h, hipMemcpyAsync(h->desc_dev, slot, h->desc_bytes, hipMemcpyHostToDevice, h->stream));
        SWARM_HIP(h, hipEventRecord(h->desc_free[slot_index], h->stream));
    }

    GossipArgs a = gossip_args(h, (uint32_t)h->round, (uint32_t)(h->round % (c.stale_max + 1)));
    SWARM_TRY(record_timing(h, h->ev_gossip, h->timed_gossip, 0));
    const bool inplace = c.apply_mode == SWARM_APPLY_INPLACE;
    if (c.codec == SWARM_CODEC_PREFIX) {
        // multi-resolution registers: pairs whose reads are both stale run node by node, all others through
        // the kernel that takes any mix (the groups are laid out as fresh/fresh, stale/stale, one stale)
        const DiagObjective *local = fused ? &h->diag : nullptr;
        GossipArgs ga = a;
        const uint32_t counts[3] = {(uint32_t)groups[0].size(), (uint32_t)groups[1].size(), (uint32_t)groups[2].size()};
        for (int gidx = 0; gidx < 3; ++gidx) {
            SWARM_HIP(h, launch_prefix(ga, local, inplace, c.lr, gidx == 1 ? 1 : 0, counts[gidx], h->stream));
            ga.pairs += counts[gidx];
        }
        SWARM_TRY(record_timing(h, h->ev_gossip, h->timed_gossip, 1));
        h->timed_gossip += 1;
        SWARM_HIP(h, launch_prefix(a, local, inplace, c.lr, 2, nsingles, h->stream));
    } else {
        if (pair_scale_policy && npairs) {   // distance of every pair first, then each pair quantizes at its own scale
            SWARM_HIP(h, hipMemsetAsync(h->linf_dev, 0, sizeof(uint32_t) * PAIR_STRIPES * npairs, h->stream));
            SWARM_HIP(h, launch_pair_linf_desc(h->X, c.d, a.pairs, npairs, h->linf_dev, h->stream));
        }
        {
            GossipArgs ga = a;
            if (pair_scale_policy) ga.pair_linf = h->linf_dev;
            for (int gidx = 0; gidx < 3; ++gidx) {
                const uint32_t count = (uint32_t)groups[gidx].size();
                    if (fused)
                    SWARM_HIP(h, launch_fused_pairs(ga, h->diag, c.bits, inplace, c.H, c.lr, group_mode[gidx], count, h->stream));
                else
                    SWARM_HIP(h, launch_gossip_pairs(ga, c.bits, delta_mode, group_mode[gidx], count, h->stream));
                ga.pairs += count;
                if (ga.pair_linf) ga.pair_linf += (size_t)count * PAIR_STRIPES;
            }
        }
        SWARM_TRY(record_timing(h, h->ev_gossip, h->timed_gossip, 1));
        h->timed_gossip += 1;
        // unmatched nodes: publish their code (needed by later stale reads) and apply their own steps
        if (fused) {
            SWARM_HIP(h, launch_fused_singles(a, h->diag, c.bits, inplace, c.H, c.lr, nsingles, h->stream));
        } else {
            const uint32_t singles_bits = pair_scale_policy ? 0u : c.bits;   // no shared scale: nothing to publish
            bool singles_work = singles_bits != 0;
            for (uint32_t u : singles) singles_work |= h->pending[u] != 0;
            if (singles_work) SWARM_HIP(h, launch_gossip_singles(a, singles_bits, nsingles, h->stream));
        }
    }

    if (c.scale_policy == SWARM_SCALE_GLOBAL_LINF)      // the disagreement this round saw sets the next round's scale
        SWARM_HIP(h, launch_scale_close(h->eps_slots_dev, h->scale_state_dev, a.slot_now, a.ring_depth, c.bits, npairs,
                                        h->stream));

    std::fill(h->pending.begin(), h->pending.end(), 0);
    h->round += 1;
    h->interactions += npairs;
    if (c.codec == SWARM_CODEC_PREFIX)      // first plane and checksums of every read; escalations are counted on the device
        h->bits_communicated += 2ull * npairs * (c.d * 4 + 64ull * ((c.d + PREFIX_TILE - 1) / PREFIX_TILE));
    else
        h->bits_communicated += 2ull * npairs * c.d * (c.bits ? c.bits : 32);
    h->prefix_tile_reads += c.codec == SWARM_CODEC_PREFIX ? 2ull * npairs * ((c.d + PREFIX_TILE - 1) / PREFIX_TILE) : 0ull;
    return SWARM_OK;
}

swarm_status swarm_gossip_round(swarm_t h, const uint32_t *pairs_host, uint32_t npairs, const uint8_t *stale_host) {
    if (!h) return SWARM_EINVAL;
    return round_impl(h, pairs_host, npairs, stale_host, false);
}

swarm_status swarm_round_fused(swarm_t h, const uint32_t *pairs_host, uint32_t npairs, const uint8_t *stale_host) {
    if (!h) return SWARM_EINVAL;
    return round_impl(h, pairs_host, npairs, stale_host, true);
}

swarm_status swarm_interact(swarm_t h, uint32_t i, uint32_t j) {
    if (!h) return SWARM_EINVAL;
    const swarm_config &c = h->cfg;
    if (c.stale_max != 0) return fail(h, SWARM_EINVAL, "Algorithm 1 steps need stale_max = 0");
    if (c.apply_mode != SWARM_APPLY_DEFERRED) return fail(h, SWARM_EINVAL, "Algorithm 1 defers the local steps");
    if (c.scale_policy != SWARM_SCALE_FIXED) return fail(h, SWARM_EINVAL, "Algorithm 1 steps use the fixed lattice scale");
    if (i >= c.n || j >= c.n || i == j ||
        !std::binary_search(h->edge_keys.begin(), h->edge_keys.end(), edge_key(i, j)))
        return fail(h, SWARM_EINVAL, "responder is not a neighbour of the initiator");
    {
        const swarm_status rc = ensure_snapshots(h);
        if (rc != SWARM_OK) return rc;
    }
    bool has_delta = h->pending[i] != 0;
    if (c.H > 0 && h->kind != OBJ_NONE) {
        SWARM_TRY(upload_nodes(h, &i, 1));
        SWARM_TRY(record_timing(h, h->ev_local, h->timed_local, 0));
        SWARM_TRY(run_local_steps(h, h->Xhat, &i, h->nodes_dev, 1, (uint32_t)h->interactions));
        SWARM_TRY(record_timing(h, h->ev_local, h->timed_local, 1));
        h->timed_local += 1;
        has_delta = true;
    }
    const GossipArgs a = gossip_args(h, (uint32_t)h->interactions, 0);
    SWARM_TRY(record_timing(h, h->ev_gossip, h->timed_gossip, 0));
    const SeqDesc one{i, j, (uint32_t)h->interactions, has_delta ? SEQ_HAS_DELTA : 0u};
    if (c.codec == SWARM_CODEC_PREFIX) SWARM_HIP(h, launch_prefix_interact(a, nullptr, one, 1, h->stream));
    else SWARM_HIP(h, launch_interact(a, c.bits, nullptr, one, 1, nullptr, c.lr, h->stream));
    SWARM_TRY(record_timing(h, h->ev_gossip, h->timed_gossip, 1));
    h->timed_gossip += 1;
    h->pending[i] = 0;
    h->interactions += 1;
    if (c.codec == SWARM_CODEC_PREFIX) {     // read by prefixes, average written back with as many bits
        const uint64_t tiles = (c.d + PREFIX_TILE - 1) / PREFIX_TILE;
        h->bits_communicated += 2ull * (c.d * 4 + 64ull * tiles);
        h->prefix_tile_reads += tiles;
    } else {
        h->bits_communicated += 2ull * c.d * (c.bits ? c.bits : 32);
    }
    return SWARM_OK;
}

// Per-interaction staging of a batch: [SeqDesc | initiator | steps | event] x capacity.
static swarm_status ensure_sequence_buffers(swarm_t h, uint32_t count) {
    if (count <= h->seq_cap) return SWARM_OK;
    count = std::max(count, std::min(SEQ_CHUNK, 1024u));
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    if (h->seq_dev) { (void)hipFree(h->seq_dev); h->seq_dev = nullptr; }
    if (h->seq_host) { (void)hipHostFree(h->seq_host); h->seq_host = nullptr; }
    h->seq_cap = 0;
    const size_t bytes = (size_t)count * SEQ_ENTRY_BYTES;
    SWARM_HIP(h, hipMalloc((void **)&h->seq_dev, bytes));
    SWARM_HIP(h, hipHostMalloc((void **)&h->seq_host, bytes, hipHostMallocDefault));
    if (!h->seq_free) {
        SWARM_HIP(h, hipEventCreateWithFlags(&h->seq_free, hipEventDisableTiming));
        SWARM_HIP(h, hipEventRecord(h->seq_free, h->stream));
    }
    h->seq_cap = count;
    return SWARM_OK;
}

swarm_status swarm_run_sequential(swarm_t h, uint32_t count, uint32_t *pairs_host, uint32_t *launches) {
    if (!h) return SWARM_EINVAL;
    const swarm_config &c = h->cfg;
    if (launches) *launches = 0;
    if (c.stale_max != 0) return fail(h, SWARM_EINVAL, "Algorithm 1 steps need stale_max = 0");
    if (c.apply_mode != SWARM_APPLY_DEFERRED) return fail(h, SWARM_EINVAL, "Algorithm 1 defers the local steps");
    if (c.scale_policy != SWARM_SCALE_FIXED) return fail(h, SWARM_EINVAL, "Algorithm 1 steps use the fixed lattice scale");
    if (h->kind == OBJ_MLP && c.steps_law != SWARM_STEPS_CONSTANT)
        return fail(h, SWARM_ESTATE, "the MLP objective takes a constant number of local steps");
    if (count == 0) return SWARM_OK;
    for (const std::vector<uint32_t> &nb : h->adj)
        if (nb.empty()) return fail(h, SWARM_ESTATE, "a node has no neighbour");
    SWARM_TRY(ensure_snapshots(h));
    const bool with_steps = c.H > 0 && h->kind != OBJ_NONE;
    // the diagonal objective is per-coordinate: its steps are taken inside the interaction kernel
    const bool steps_inside = with_steps && h->kind == OBJ_DIAG && c.codec == SWARM_CODEC_FIXED;
    // small least-squares models: one workgroup runs an initiator's steps and then its interaction
    const bool lsq_inside = with_steps && h->kind == OBJ_LSQ && c.codec == SWARM_CODEC_FIXED && h->lsq.part != nullptr;
    const uint64_t tiles = (c.d + PREFIX_TILE - 1) / PREFIX_TILE;
    const GossipArgs a = gossip_args(h, 0, 0);
    uint32_t total_launches = 0;
    SWARM_TRY(record_timing(h, h->ev_gossip, h->timed_gossip, 0));
    std::vector<uint32_t> level_of, last_level(c.n), order, level_start;
    for (uint32_t done = 0; done < count;) {
        const uint32_t m = std::min(count - done, SEQ_CHUNK);
        SWARM_TRY(ensure_sequence_buffers(h, m));
        // 1. the pairs Algorithm 1 draws next, and the earliest launch each interaction can join: one
        //    after the last launch that touches either of its nodes (interactions on disjoint nodes commute).
        level_of.assign(m, 0);
        std::fill(last_level.begin(), last_level.end(), 0u);
        std::vector<SeqDesc> drawn(m);
        uint32_t levels = 0;
        for (uint32_t t = 0; t < m; ++t) {
            const uint32_t event = (uint32_t)(h->interactions + t);
            const Words4 w = stream(c.seed, TAG_PICK, 0, 0, event, 0);
            const uint32_t i = scaled_index(w.w0, c.n);
            const std::vector<uint32_t> &nb = h->adj[i];
            const uint32_t j = nb[scaled_index(w.w1, (uint32_t)nb.size())];
            const bool has_delta = with_steps || h->pending[i];
            h->pending[i] = 0;
            const uint32_t steps = with_steps ? draw_steps(c, i, event) : 0u;
            drawn[t] = SeqDesc{i, j, event, (has_delta ? SEQ_HAS_DELTA : 0u) | (steps << 8)};
            const uint32_t level = std::max(last_level[i], last_level[j]) + 1;
            last_level[i] = last_level[j] = level;
            level_of[t] = level - 1;
            levels = std::max(levels, level);
            if (pairs_host) { pairs_host[2 * (size_t)(done + t)] = i; pairs_host[2 * (size_t)(done + t) + 1] = j; }
        }
        // 2. interactions grouped by launch, in their own order inside a launch
        level_start.assign(levels + 1, 0);
        for (uint32_t t = 0; t < m; ++t) level_start[level_of[t] + 1] += 1;
        for (uint32_t l = 0; l < levels; ++l) level_start[l + 1] += level_start[l];
        order.assign(level_start.begin(), level_start.end() - 1);
        SWARM_HIP(h, hipEventSynchronize(h->seq_free));
        SeqDesc *descs = (SeqDesc *)h->seq_host;
        uint32_t *ids = (uint32_t *)(h->seq_host + (size_t)h->seq_cap * sizeof(SeqDesc));
        uint32_t *steps = ids + h->seq_cap, *events = steps + h->seq_cap;
        for (uint32_t t = 0; t < m; ++t) {
            const uint32_t at = order[level_of[t]]++;
            descs[at] = drawn[t];
            ids[at] = drawn[t].ni;
            steps[at] = drawn[t].flags >> 8;
            events[at] = drawn[t].event;
        }
        SWARM_HIP(h, hipMemcpyAsync(h->seq_dev, h->seq_host, (size_t)h->seq_cap * SEQ_ENTRY_BYTES, hipMemcpyHostToDevice,
                                    h->stream));
        SWARM_HIP(h, hipEventRecord(h->seq_free, h->stream));
        const SeqDesc *descs_dev = (const SeqDesc *)h->seq_dev;
        const uint32_t *ids_dev = (const uint32_t *)(h->seq_dev + (size_t)h->seq_cap * sizeof(SeqDesc));
        // 3. one launch per group (preceded by the initiators' local steps where they are a kernel of their own)
        for (uint32_t l = 0; l < levels; ++l) {
            const uint32_t off = level_start[l], width = level_start[l + 1] - off;
            if (lsq_inside) {
                SWARM_HIP(h, launch_lsq_interact(a, c.bits, descs_dev + off, width, h->lsq, c.lr, h->stream));
                continue;
            }
            if (with_steps && !steps_inside) {
                LocalSlots slots;
                slots.nodes = ids_dev + off;
                slots.steps = c.steps_law == SWARM_STEPS_CONSTANT ? nullptr : ids_dev + h->seq_cap + off;
                slots.events = ids_dev + 2 * (size_t)h->seq_cap + off;
                SWARM_TRY(launch_local(h, h->Xhat, slots, width, 0));
            }
            if (c.codec == SWARM_CODEC_PREFIX)
                SWARM_HIP(h, launch_prefix_interact(a, descs_dev + off, SeqDesc{}, width, h->stream));
            else
                SWARM_HIP(h, launch_interact(a, c.bits, descs_dev + off, SeqDesc{}, width, steps_inside ? &h->diag : nullptr,
                                             c.lr, h->stream));
        }
        total_launches += levels;
        h->interactions += m;
        if (c.codec == SWARM_CODEC_PREFIX) {
            h->bits_communicated += (uint64_t)m * 2ull * (c.d * 4 + 64ull * tiles);
            h->prefix_tile_reads += (uint64_t)m * tiles;
        } else {
            h->bits_communicated += (uint64_t)m * 2ull * c.d * (c.bits ? c.bits : 32);
        }
        done += m;
    }
    SWARM_TRY(record_timing(h, h->ev_gossip, h->timed_gossip, 1));
    h->timed_gossip += 1;
    if (launches) *launches = total_launches;
    return SWARM_OK;
}

swarm_status swarm_quantize(const float *x_dev, uint64_t d, float eps, uint32_t bits, uint64_t seed, uint32_t node,
                            uint32_t event, void *codes_dev, void *hip_stream) {
    if (!x_dev || !codes_dev || d == 0 || d % 8 != 0 || !valid_bits(bits) || !(eps > 0.f))
        return fail(nullptr, SWARM_EINVAL, "quantize: bad argument");
    if (((uintptr_t)x_dev & 15u) || ((uintptr_t)codes_dev & 7u))
        return fail(nullptr, SWARM_EINVAL, "quantize: x_dev must be 16-byte aligned and codes_dev 8-byte aligned");
    const hipError_t e = launch_quantize(x_dev, d, eps, 1.0f / eps, bits, seed, node, event, (uint8_t *)codes_dev,
                                         nullptr, (hipStream_t)hip_stream);
    return e == hipSuccess ? SWARM_OK : fail(nullptr, SWARM_EDEVICE, hipGetErrorString(e));
}

swarm_status swarm_dequantize(const void *codes_dev, const float *key_dev, uint64_t d, float eps, uint32_t bits,
                              float *out_dev, void *hip_stream) {
    if (!codes_dev || !key_dev || !out_dev || d == 0 || d % 8 != 0 || !valid_bits(bits) || !(eps > 0.f))
        return fail(nullptr, SWARM_EINVAL, "dequantize: bad argument");
    if (((uintptr_t)key_dev & 15u) || ((uintptr_t)out_dev & 15u) || ((uintptr_t)codes_dev & 7u))
        return fail(nullptr, SWARM_EINVAL, "dequantize: key_dev and out_dev must be 16-byte aligned and codes_dev 8-byte aligned");
    const hipError_t e = launch_dequantize((const uint8_t *)codes_dev, key_dev, d, eps, 1.0f / eps, bits, out_dev,
                                           (hipStream_t)hip_stream);
    return e == hipSuccess ? SWARM_OK : fail(nullptr, SWARM_EDEVICE, hipGetErrorString(e));
}

static float *matrix_of(swarm_t h, uint32_t which) {
    switch (which) {
        case SWARM_MODELS_COMM: return h->X;
        case SWARM_MODELS_LIVE: return h->W;
        case SWARM_MODELS_SNAP: return h->Xhat;
        default: return nullptr;
    }
}

static swarm_status check_window(swarm_t h, uint32_t which, uint32_t node0, uint32_t count, uint64_t k0, uint64_t len,
                                 const void *host) {
    if (which > SWARM_MODELS_SNAP) return fail(h, SWARM_EINVAL, "unknown model matrix");
    if (which == SWARM_MODELS_SNAP) {
        const swarm_status rc = ensure_snapshots(h);
        if (rc != SWARM_OK) return rc;
    }
    if (!host || count == 0 || len == 0 || (uint64_t)node0 + count > h->cfg.n || k0 + len > h->cfg.d)
        return fail(h, SWARM_EINVAL, "window out of range");
    return SWARM_OK;
}

swarm_status swarm_read_models(swarm_t h, uint32_t which, uint32_t node0, uint32_t count, uint64_t k0, uint64_t len,
                               float *dst_host) {
    if (!h) return SWARM_EINVAL;
    const swarm_status rc = check_window(h, which, node0, count, k0, len, dst_host);
    if (rc != SWARM_OK) return rc;
    const float *src = matrix_of(h, which) + (uint64_t)node0 * h->cfg.d + k0;
    SWARM_HIP(h, hipMemcpy2DAsync(dst_host, len * sizeof(float), src, h->cfg.d * sizeof(float), len * sizeof(float),
                                  count, hipMemcpyDeviceToHost, h->stream));
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    return SWARM_OK;
}

swarm_status swarm_write_models(swarm_t h, uint32_t which, uint32_t node0, uint32_t count, uint64_t k0, uint64_t len,
                                const float *src_host) {
    if (!h) return SWARM_EINVAL;
    const swarm_status rc = check_window(h, which, node0, count, k0, len, src_host);
    if (rc != SWARM_OK) return rc;
    float *dst = matrix_of(h, which) + (uint64_t)node0 * h->cfg.d + k0;
    SWARM_HIP(h, hipMemcpy2DAsync(dst, h->cfg.d * sizeof(float), src_host, len * sizeof(float), len * sizeof(float),
                                  count, hipMemcpyHostToDevice, h->stream));
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    if (which == SWARM_MODELS_LIVE && h->cfg.apply_mode == SWARM_APPLY_DEFERRED)
        for (uint32_t u = node0; u < node0 + count; ++u) h->pending[u] = 1;
    if (which == SWARM_MODELS_COMM) for (uint32_t u = node0; u < node0 + count; ++u) h->pending[u] = 0;
    return SWARM_OK;
}

// ---- exact resume -----------------------------------------------------------------------------
// Every random draw is a function of (seed, round or interaction number, ids), so the models, the
// registers, the counters and a few integers are the whole state of a run.
namespace {

struct StateHeader {
    uint64_t magic, d, seed, round, interactions, bits_communicated, prefix_tile_reads;
    uint32_t version, n, bits, stale_max, apply_mode, codec, scale_policy, has_snapshots;
    float eps;
    uint32_t pad;
};
constexpr uint64_t STATE_MAGIC = 0x31657461745377ull;   // "wStatE1" little-endian, zero-padded

struct StatePart { void *dev; size_t bytes; };

// Device blocks of a state image, in order; `snapshots` as in the image being written or read.
void state_parts(swarm_t h, bool snapshots, std::vector<StatePart> &parts) {
    const swarm_config &c = h->cfg;
    const size_t model_bytes = (size_t)c.n * c.d * sizeof(float);
    parts.clear();
    parts.push_back({h->X, model_bytes});
    if (c.apply_mode == SWARM_APPLY_DEFERRED) parts.push_back({h->W, model_bytes});
    if (snapshots) parts.push_back({h->Xhat, model_bytes});
    if (c.bits) parts.push_back({h->ring, (size_t)(c.stale_max + 1) * c.n * h->row_bytes});
    parts.push_back({h->counters_dev, sizeof(DeviceCounters)});
    if (h->prefix_stats_dev) parts.push_back({h->prefix_stats_dev, sizeof(PrefixStats) * PREFIX_STRIPES});
    if (h->eps_slots_dev) {
        parts.push_back({h->eps_slots_dev, sizeof(float) * (c.stale_max + 1)});
        parts.push_back({h->scale_state_dev, sizeof(uint32_t) * (2 + FAR_STRIPES)});
    }
}

uint64_t state_size(swarm_t h, bool snapshots) {
    uint64_t total = sizeof(StateHeader) + ((h->cfg.n + 7u) & ~7u);
    std::vector<StatePart> parts;
    state_parts(h, snapshots, parts);
    for (const StatePart &p : parts) total += (p.bytes + 7u) & ~(size_t)7u;
    return total;
}

}  // namespace

swarm_status swarm_state_bytes(swarm_t h, uint64_t *nbytes) {
    if (!h || !nbytes) return SWARM_EINVAL;
    *nbytes = state_size(h, h->Xhat != nullptr);
    return SWARM_OK;
}

swarm_status swarm_save_state(swarm_t h, void *dst_host, uint64_t nbytes) {
    if (!h) return SWARM_EINVAL;
    const bool snapshots = h->Xhat != nullptr;
    if (!dst_host || nbytes < state_size(h, snapshots)) return fail(h, SWARM_EINVAL, "state buffer missing or too small");
    const swarm_config &c = h->cfg;
    StateHeader hd{};
    hd.magic = STATE_MAGIC; hd.version = 1;
    hd.d = c.d; hd.seed = c.seed; hd.n = c.n; hd.bits = c.bits; hd.stale_max = c.stale_max;
    hd.apply_mode = c.apply_mode; hd.codec = c.codec; hd.scale_policy = c.scale_policy; hd.eps = c.eps;
    hd.has_snapshots = snapshots;
    hd.round = h->round; hd.interactions = h->interactions; hd.bits_communicated = h->bits_communicated;
    hd.prefix_tile_reads = h->prefix_tile_reads;
    uint8_t *out = (uint8_t *)dst_host;
    std::memcpy(out, &hd, sizeof(hd));
    out += sizeof(hd);
    std::memset(out, 0, (c.n + 7u) & ~7u);
    std::memcpy(out, h->pending.data(), c.n);
    out += (c.n + 7u) & ~7u;
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    std::vector<StatePart> parts;
    state_parts(h, snapshots, parts);
    for (const StatePart &p : parts) {
        SWARM_HIP(h, hipMemcpy(out, p.dev, p.bytes, hipMemcpyDeviceToHost));
        out += (p.bytes + 7u) & ~(size_t)7u;
    }
    return SWARM_OK;
}

swarm_status swarm_load_state(swarm_t h, const void *src_host, uint64_t nbytes) {
    if (!h) return SWARM_EINVAL;
    if (!src_host || nbytes < sizeof(StateHeader)) return fail(h, SWARM_EINVAL, "state image missing or truncated");
    const swarm_config &c = h->cfg;
    StateHeader hd;
    std::memcpy(&hd, src_host, sizeof(hd));
    if (hd.magic != STATE_MAGIC || hd.version != 1) return fail(h, SWARM_EINVAL, "not a state image of this library version");
    if (hd.n != c.n || hd.d != c.d || hd.bits != c.bits || hd.stale_max != c.stale_max || hd.apply_mode != c.apply_mode ||
        hd.codec != c.codec || hd.scale_policy != c.scale_policy || hd.seed != c.seed || hd.eps != c.eps)
        return fail(h, SWARM_EINVAL, "state image belongs to a swarm of another configuration");
    if (hd.has_snapshots) SWARM_TRY(ensure_snapshots(h));
    if (nbytes < state_size(h, hd.has_snapshots != 0)) return fail(h, SWARM_EINVAL, "state image truncated");
    const uint8_t *in = (const uint8_t *)src_host + sizeof(hd);
    h->pending.assign(in, in + c.n);
    in += (c.n + 7u) & ~7u;
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    std::vector<StatePart> parts;
    state_parts(h, hd.has_snapshots != 0, parts);
    for (const StatePart &p : parts) {
        SWARM_HIP(h, hipMemcpy(p.dev, in, p.bytes, hipMemcpyHostToDevice));
        in += (p.bytes + 7u) & ~(size_t)7u;
    }
    if (!hd.has_snapshots && h->Xhat)     // saved before any step of Algorithm 1: the snapshots still equalled the models
        SWARM_HIP(h, hipMemcpy(h->Xhat, h->X, (size_t)c.n * c.d * sizeof(float), hipMemcpyDeviceToDevice));
    h->round = hd.round; h->interactions = hd.interactions; h->bits_communicated = hd.bits_communicated;
    h->prefix_tile_reads = hd.prefix_tile_reads;
    h->match_round = ~0ull;          // a matching enqueued for the old round counter is of no use now
    return SWARM_OK;
}

swarm_status swarm_models_ptr(swarm_t h, uint32_t which, float **ptr_dev) {
    if (!h) return SWARM_EINVAL;
    if (!ptr_dev || which > SWARM_MODELS_SNAP) return fail(h, SWARM_EINVAL, "unknown model matrix");
    if (which == SWARM_MODELS_SNAP) {
        const swarm_status rc = ensure_snapshots(h);
        if (rc != SWARM_OK) return rc;
    }
    *ptr_dev = matrix_of(h, which);
    return SWARM_OK;
}

swarm_status swarm_read_codes(swarm_t h, uint32_t age, uint32_t node, uint64_t byte0, uint64_t len,
                              uint8_t *dst_host) {
    if (!h) return SWARM_EINVAL;
    const swarm_config &c = h->cfg;
    if (!c.bits) return fail(h, SWARM_ESTATE, "no codes with bits = 0");
    if (!dst_host || node >= c.n || age > c.stale_max || byte0 + len > h->row_bytes || len == 0)
        return fail(h, SWARM_EINVAL, "code window out of range");
    // the last completed event wrote slot (round-1) mod depth in round mode; Algorithm 1 steps write slot 0
    const uint64_t depth = c.stale_max + 1;
    const uint64_t last = h->round ? (h->round - 1) % depth : 0;
    const uint64_t slot = (last + depth - age) % depth;
    const uint8_t *src = h->ring + (slot * c.n + node) * h->row_bytes + byte0;
    SWARM_HIP(h, hipMemcpyAsync(dst_host, src, len, hipMemcpyDeviceToHost, h->stream));
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    return SWARM_OK;
}

swarm_status swarm_potential(swarm_t h, double *gamma_host, float *mu_dev) {
    if (!h) return SWARM_EINVAL;
    if (!gamma_host) return fail(h, SWARM_EINVAL, "null output");
    SWARM_HIP(h, launch_potential(h->X, h->cfg.n, h->cfg.d, mu_dev, h->partials_dev, potential_partials(h->cfg.d),
                                  h->gamma_dev, h->stream));
    SWARM_HIP(h, hipMemcpyAsync(h->scalar_host, h->gamma_dev, sizeof(double), hipMemcpyDeviceToHost, h->stream));
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    *gamma_host = *h->scalar_host;
    return SWARM_OK;
}

swarm_status swarm_scale(swarm_t h, float *eps_next, float *disagreement) {
    if (!h) return SWARM_EINVAL;
    uint32_t state[2] = {0u, 0u};
    std::memcpy(&state[0], &h->cfg.eps, sizeof(float));
    if (h->scale_state_dev) {
        SWARM_HIP(h, hipStreamSynchronize(h->stream));
        SWARM_HIP(h, hipMemcpy(state, h->scale_state_dev, sizeof(state), hipMemcpyDeviceToHost));
    }
    if (eps_next) std::memcpy(eps_next, &state[0], sizeof(float));
    if (disagreement) std::memcpy(disagreement, &state[1], sizeof(float));
    return SWARM_OK;
}

swarm_status swarm_pair_linf(swarm_t h, const uint32_t *pairs_host, uint32_t npairs, float *linf_host) {
    if (!h) return SWARM_EINVAL;
    if (!pairs_host || !linf_host || npairs == 0 || npairs > h->cfg.n / 2)
        return fail(h, SWARM_EINVAL, "pair list out of range");
    for (uint32_t k = 0; k < 2 * npairs; ++k)
        if (pairs_host[k] >= h->cfg.n) return fail(h, SWARM_EINVAL, "pair endpoint out of range");
    SWARM_TRY(upload_nodes(h, pairs_host, 2 * npairs));
    SWARM_HIP(h, hipMemsetAsync(h->linf_dev, 0, sizeof(uint32_t) * PAIR_STRIPES * npairs, h->stream));
    SWARM_HIP(h, launch_pair_linf(h->X, h->cfg.d, h->nodes_dev, npairs, h->linf_dev, h->stream));
    std::vector<uint32_t> stripes((size_t)npairs * PAIR_STRIPES);
    SWARM_HIP(h, hipMemcpyAsync(stripes.data(), h->linf_dev, sizeof(uint32_t) * stripes.size(), hipMemcpyDeviceToHost, h->stream));
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    for (uint32_t p = 0; p < npairs; ++p) {          // non-negative floats order like their bit patterns
        const uint32_t bits = *std::max_element(stripes.begin() + (size_t)p * PAIR_STRIPES, stripes.begin() + (size_t)(p + 1) * PAIR_STRIPES);
        std::memcpy(linf_host + p, &bits, sizeof(float));
    }
    return SWARM_OK;
}

// Sum of the striped escalation counts (synchronises; zeros without multi-resolution registers).
static swarm_status prefix_totals(swarm_t h, PrefixStats *total) {
    *total = PrefixStats{};
    if (!h->prefix_stats_dev) return SWARM_OK;
    std::vector<PrefixStats> stripes(PREFIX_STRIPES);
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    SWARM_HIP(h, hipMemcpy(stripes.data(), h->prefix_stats_dev, sizeof(PrefixStats) * PREFIX_STRIPES, hipMemcpyDeviceToHost));
    for (const PrefixStats &s : stripes) {
        for (int l = 0; l < 2; ++l) {
            total->tiles[l] += s.tiles[l];
            total->coords[l] += s.coords[l];
            total->written_back[l] += s.written_back[l];
        }
        total->unconfirmed += s.unconfirmed;
    }
    return SWARM_OK;
}

swarm_status swarm_counters(swarm_t h, uint64_t *rounds, uint64_t *interactions, uint64_t *bits_communicated,
                            uint64_t *decode_failures) {
    if (!h) return SWARM_EINVAL;
    DeviceCounters *dc = (DeviceCounters *)h->scalar_host;
    SWARM_HIP(h, hipMemcpyAsync(dc, h->counters_dev, sizeof(DeviceCounters), hipMemcpyDeviceToHost, h->stream));
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    if (rounds) *rounds = h->round;
    if (interactions) *interactions = h->interactions;
    if (bits_communicated) {   // escalated tiles read 4 (to 8 bits) or 12 (to 16 bits) more bits per coordinate
        PrefixStats total;
        SWARM_TRY(prefix_totals(h, &total));
        *bits_communicated = h->bits_communicated + 4ull * (total.coords[0] + total.written_back[0]) +
                             12ull * (total.coords[1] + total.written_back[1]);
    }
    if (decode_failures) *decode_failures = dc->decode_failures;
    if (dc->barrier_timeouts)
        return fail(h, SWARM_EDEVICE, "least-squares local steps: a workgroup timed out waiting for the others of its node");
    if (dc->range_clamped) return fail(h, SWARM_ERANGE, "|x/eps| reached the clamp 2^29");
    return SWARM_OK;
}

swarm_status swarm_prefix_stats(swarm_t h, uint64_t *tiles, uint64_t *unconfirmed) {
    if (!h) return SWARM_EINVAL;
    PrefixStats total;
    SWARM_TRY(prefix_totals(h, &total));
    if (tiles) {
        tiles[1] = total.tiles[0];
        tiles[2] = total.tiles[1];
        tiles[0] = h->prefix_tile_reads - tiles[1] - tiles[2];
    }
    if (unconfirmed) *unconfirmed = total.unconfirmed;
    return SWARM_OK;
}

swarm_status swarm_stream_copy(void *dst_dev, const void *src_dev, uint64_t nbytes, void *hip_stream) {
    if (!dst_dev || !src_dev || nbytes == 0 || nbytes % 16 != 0 || nbytes > (1ull << 36))
        return fail(nullptr, SWARM_EINVAL, "stream copy: size must be a multiple of 16, at most 2^36");
    const hipError_t e = launch_stream_copy(src_dev, dst_dev, nbytes, (hipStream_t)hip_stream);
    return e == hipSuccess ? SWARM_OK : fail(nullptr, SWARM_EDEVICE, hipGetErrorString(e));
}

swarm_status swarm_stream_mix(void *dst_dev, const void *src_dev, uint64_t stream_bytes, uint32_t n_read,
                              uint32_t n_write, void *hip_stream) {
    if (!dst_dev || !src_dev || stream_bytes == 0 || stream_bytes % 16 != 0 || stream_bytes > (1ull << 36))
        return fail(nullptr, SWARM_EINVAL, "stream mix: size must be a multiple of 16, at most 2^36");
    const hipError_t e = launch_stream_mix(src_dev, dst_dev, stream_bytes, n_read, n_write, (hipStream_t)hip_stream);
    if (e == hipErrorInvalidValue) return fail(nullptr, SWARM_EINVAL, "stream mix: unsupported (n_read, n_write)");
    return e == hipSuccess ? SWARM_OK : fail(nullptr, SWARM_EDEVICE, hipGetErrorString(e));
}

swarm_status swarm_timing_reset(swarm_t h) {
    if (!h) return SWARM_EINVAL;
    h->timed_gossip = h->timed_local = 0;
    h->timing_armed = true;
    return SWARM_OK;
}

swarm_status swarm_kernel_times(swarm_t h, double *gossip_ms, uint32_t *gossip_calls, double *local_ms,
                                uint32_t *local_calls) {
    if (!h) return SWARM_EINVAL;
    SWARM_HIP(h, hipStreamSynchronize(h->stream));
    auto total = [&](const std::vector<hipEvent_t> &ev, uint32_t calls, double *ms, uint32_t *count) -> swarm_status {
        const uint32_t recorded = std::min(calls, MAX_TIMED_CALLS);
        double sum = 0.0;
        for (uint32_t k = 0; k < recorded; ++k) {
            float t = 0.f;
            SWARM_HIP(h, hipEventElapsedTime(&t, ev[2 * k], ev[2 * k + 1]));
            sum += t;
        }
        if (ms) *ms = sum;
        if (count) *count = recorded;
        return SWARM_OK;
    };
    SWARM_TRY(total(h->ev_gossip, h->timed_gossip, gossip_ms, gossip_calls));
    SWARM_TRY(total(h->ev_local, h->timed_local, local_ms, local_calls));
    return SWARM_OK;
}

}  // extern "C"
