/*
 * swarm.h -- C ABI of the MI355X swarm-interaction library.
 *
 * One handle simulates the n nodes of SwarmSGD (arXiv 1910.12308) on one GPU: every
 * node's model is a row of an n x d float32 matrix in device memory.  The calls are
 * the steps of one swarm interaction as the paper states them: n >= 2 nodes on a
 * communication graph G, pairwise interactions, H local SGD steps that are computed
 * but not yet applied, b-bit quantized exchange decoded against the receiver's own
 * model, and non-blocking (possibly stale) reads of the partner's buffer
 * (Section 2 "The Distributed System Model", Section 3, Algorithm 1, Corollary 2.1).
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses.
 *   - The handle OWNS the model matrices X (current / communicated), W (live copy with
 *     the pending local steps), Xhat (model at the node's last initiation, created as a
 *     copy of X on first use), and the ring of packed code rows.  Objective data
 *     passed to swarm_set_objective_* is BORROWED: it must outlive the handle.
 *   - Host arrays are only read (or written) during the call.
 *   - Kernels are enqueued on the HIP stream given at swarm_init.  Calls return after
 *     enqueueing, except those documented as synchronising.
 *   - Every call returns a swarm_status; nothing throws or aborts across the ABI.
 *     swarm_last_error() gives the text of the last failure on a handle.
 *   - One host thread per handle; calls on one handle must not overlap.
 */
#ifndef SWARM_H
#define SWARM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct swarm_ctx *swarm_t;

typedef enum {
    SWARM_OK = 0,
    SWARM_EINVAL = 1,   /* bad argument: not an edge of G, node repeated, size, bits ...  */
    SWARM_ENOMEM = 2,   /* device or host allocation failed                               */
    SWARM_EDEVICE = 3,  /* a HIP call failed                                              */
    SWARM_ESTATE = 4,   /* call not valid in the handle's state (e.g. no objective set)   */
    SWARM_ERANGE = 5    /* reported by swarm_counters: |x/eps| reached the clamp 2^29, or a
                           coordinate was not a number                                    */
} swarm_status;

/* When the local steps reach the exchanged model.  DEFERRED (the paper: the node computes its
 * local gradients, holds them back, averages the quantized models, then adds the
 * summed update to the average): X is exchanged, W = X - eta h~ lives in a second matrix.
 * INPLACE: the local steps update the exchanged model directly and the averaging acts on the
 * updated models; one matrix, no pending update (W is an alias of X). */
enum { SWARM_APPLY_DEFERRED = 0, SWARM_APPLY_INPLACE = 1 };

/* How the lattice scale eps is chosen.  FIXED: cfg.eps for every exchange (Corollary 2.1 fixes
 * eps up front).  PAIR_LINF: the case where the writer knows its distance to the decoding key
 * (proof of Corollary 2.1): before the exchange a reduction computes m = max_k |X_i[k] - X_j[k]|
 * for every matched pair, and the pair uses eps_ij = the smallest power of two >= m / (2^(b-1) - 3)
 * (at least 2^-100), which puts the pair inside the decoding radius, so no decode can fail.
 * Needs bits >= 4, stale_max = 0 and swarm_gossip_round (not the one-pass round or Algorithm 1);
 * unmatched nodes publish no code.
 * GLOBAL_LINF: the case where the writer does not know who will read its code, or when (appendix,
 * quantization: second case) -- with a fixed number of bits the scale has to follow the swarm.
 * One scale eps_r per round, kept with the ring slot its codes are written to; a reader decodes a
 * code of age s on the lattice eps_(r-s) Z it was written on and averages the two lattice points each
 * at its own scale, X_i' = (eps_r z_i + eps_(r-s) z_j') / 2 + pending update.  Every exchange also
 * reports max_k |X_i[k] - eps_(r-s) z_j'[k]|; with m the largest over the round,
 * eps_(r+1) = max(smallest power of two >= 2 m / (2^(b-1) - 3), eps_r / 2), and eps_(r+1) = eps_r
 * after a round without pairs.  A wrapped decode reads as a distance of about the decoding radius,
 * so a scale that is too small grows fourfold per round until decoding succeeds; no extra pass over
 * the models and no host round trip.  cfg.eps is the first round's scale and must be a power of two;
 * needs bits >= 8 (the max-norm rule would make a 4-bit lattice coarser than the typical disagreement,
 * and the rounding noise then feeds the very disagreement the scale is sized from: measured to
 * diverge); works with stale reads, both apply modes and the one-pass round, not Algorithm 1. */
enum { SWARM_SCALE_FIXED = 0, SWARM_SCALE_PAIR_LINF = 1, SWARM_SCALE_GLOBAL_LINF = 2 };

/* What a register holds and how much of it a reader fetches.  FIXED: b = cfg.bits bits per
 * coordinate, all of them read.  PREFIX: multi-resolution registers (proof of Corollary 2.1, second
 * case: the writer does not know its reader's key, so it writes the code for every resolution into
 * its own register; item 3 of the corollary: a reader needs only a prefix whose length grows with
 * log(|x - y| / eps)).  The register row holds the 16 low bits of every lattice coordinate as three
 * planes -- bits 0-3 (d/2 bytes), bits 4-7 (d/2 bytes), bits 8-15 (d bytes) -- followed by one
 * 64-bit checksum per tile of 512 coordinates: two uint32 sums s_f = sum_j (z_j mod 2^32) w_f(j)
 * mod 2^32, j the position in the tile, with the odd weights  x = (2j+1) 0x9E3779B1; x ^= x >> 15;
 * x *= 0x85EBCA6B; x ^= x >> 13; w_1 = x | 1;  y = x 0xC2B2AE35; y ^= y >> 16; w_2 = y | 1.
 * A reader decodes a tile from 4 bits, then 8, then 16, and stops
 * at the first level whose decoded tile has the writer's checksum (the confirmation that the
 * interactive protocol gets from the receiver's reply); a tile that no level confirms keeps the
 * 16-bit decode and is counted.  Needs bits = 16 and the fixed scale.  In a step of Algorithm 1 the
 * initiator reads the responder's register this way and writes the average back with as many bits
 * per tile as the read took (by then it knows its distance to the responder's key: the proof's first
 * case); bits_communicated counts both. */
enum { SWARM_CODEC_FIXED = 0, SWARM_CODEC_PREFIX = 1 };

/* Number of local steps per interaction.  CONSTANT: H for every node (the paper's experiments).
 * GEOMETRIC: each node draws H_i >= 1 afresh for every interaction from a geometric law of mean H
 * (Section 3 "Sequential model": approximates activation by independent Poisson clocks), capped
 * at 255; H_i = 1 + number of failures before the first 32-bit word below floor(2^32 / H). */
enum { SWARM_STEPS_CONSTANT = 0, SWARM_STEPS_GEOMETRIC = 1 };

enum { SWARM_MODELS_COMM = 0,  /* X: current / communicated models                        */
       SWARM_MODELS_LIVE = 1,  /* W: live copies carrying the pending local steps         */
       SWARM_MODELS_SNAP = 2   /* Xhat: models at the last initiation (Algorithm 1)       */ };

/* Problem statement (Section 2; Section 3 "Sequential model"; Corollary 2.1 parameters). */
typedef struct {
    uint32_t n;             /* number of nodes, 2 .. 4096 (the round's matching runs in one
                               workgroup that keeps the node states in its local memory)   */
    uint64_t d;             /* model dimension, a positive multiple of 8                   */
    uint32_t n_edges;       /* edges of the undirected simple graph G, at most 2^20          */
    const uint32_t *edges;  /* host, 2*n_edges endpoints (u, v), u != v; copied at init    */
    uint32_t bits;          /* b: code width, one of 0 (Q = identity, Corollary 4.2),
                               2, 4, 8, 16                                                 */
    float eps;              /* lattice scale eps > 0 (ignored when bits = 0)               */
    uint32_t H;             /* local SGD steps per interaction (constant, as in the
                               paper's experiments), 0..255                                */
    float lr;               /* learning rate eta                                           */
    uint32_t stale_max;     /* S: a read may use the partner's code from up to S rounds
                               ago; the ring keeps S+1 slots. Must be 0 when bits = 0.     */
    uint64_t seed;          /* key of every random stream                                  */
    uint32_t apply_mode;    /* SWARM_APPLY_DEFERRED (default) or SWARM_APPLY_INPLACE           */
    uint32_t steps_law;     /* SWARM_STEPS_CONSTANT (default) or SWARM_STEPS_GEOMETRIC (H >= 1;
                               not available with the MLP objective)                           */
    uint32_t scale_policy;  /* SWARM_SCALE_FIXED (default), _PAIR_LINF or _GLOBAL_LINF         */
    uint32_t codec;         /* SWARM_CODEC_FIXED (default) or SWARM_CODEC_PREFIX (bits = 16)   */
} swarm_config;

/* Create a handle.  x0_dev: d floats (device) copied into every node's model, or NULL
 * for zeros (all nodes start from the same model: Algorithm 1, initial models; the
 * registers initially hold zero vectors).  hip_stream: a hipStream_t (NULL = default
 * stream).  Allocates (2 n d) floats (n d in INPLACE mode) + (S+1) n d b/8 bytes of device
 * memory.
 * Synchronises the stream. */
swarm_status swarm_init(const swarm_config *cfg, const float *x0_dev, void *hip_stream,
                        swarm_t *out);
swarm_status swarm_destroy(swarm_t h);

/* Node objectives f_i (the paper needs only unbiased stochastic gradients with bounded
 * variance: Section 2 "Stochastic Optimization").  Data are n-major device arrays.
 *  diag: f_i(x) = 1/2 sum_k a_ik (x_k - c_ik)^2, gradient + sigma N(0, I);  a, c: n x d.
 *  lsq : f_i(x) = 1/2 |A_i x - b_i|^2, A: n x m_rows x d, b: n x m_rows; each step draws
 *        `batch` rows uniformly with replacement and scales by m_rows / batch
 *        (batch a multiple of 4, at most 64).
 *  mlp : d = hid*in + hid + out*hid + out (W1 row-major hid x in, b1, W2 out x hid, b2),
 *        ReLU, softmax cross-entropy averaged over `batch` samples of a Gaussian mixture:
 *        class y ~ label_cdf[node] (n x out float32 CDF rows), features
 *        class_means[y] (out x in) + data_sigma N(0, I).  in, hid, out, batch are
 *        multiples of 32.  Allocates activation workspace for all n nodes. */
swarm_status swarm_set_objective_diag(swarm_t h, const float *a_dev, const float *c_dev,
                                      float sigma);
swarm_status swarm_set_objective_lsq(swarm_t h, const float *A_dev, const float *b_dev,
                                     uint32_t m_rows, uint32_t batch);
swarm_status swarm_set_objective_mlp(swarm_t h, uint32_t n_in, uint32_t n_hid, uint32_t n_out,
                                     const float *class_means_dev, const float *label_cdf_dev,
                                     float data_sigma, uint32_t batch);

/* How the GEMMs of the MLP objective's local steps are computed.  FP32 (default): float32 matrix
 * instructions, float32 accumulation.  BF16X3: every float32 operand x is split into hi = bf16(x) and
 * lo = bf16(x - hi) on the fly and a product a b is taken as a_hi b_hi + a_hi b_lo + a_lo b_hi on the
 * bf16 matrix cores, float32 accumulation; the dropped terms are below 2^-16 |a b| per product, well
 * inside the 1e-4 bound of the GEMM-based gradients, and the local steps run at the speed of their
 * memory traffic instead of the float32 matrix rate.  Models, activations and updates stay float32 in
 * memory.  Call after swarm_set_objective_mlp (SWARM_ESTATE otherwise). */
enum { SWARM_MLP_FP32 = 0, SWARM_MLP_BF16X3 = 1 };
swarm_status swarm_set_mlp_arithmetic(swarm_t h, uint32_t arithmetic);

/* Local steps (Section 3 "The Communication Procedure"; appendix, definition of
 * h~_i^q): for q = 1..H, w <- w - eta g~_i(w) starting from the node's current model X_i,
 * result stored in W_i and marked pending (computed, applied only after the averaging).
 * nodes: host array of `count` distinct node ids, or NULL for all nodes. */
swarm_status swarm_local_steps(swarm_t h, const uint32_t *nodes, uint32_t count);

/* Local steps computed outside the library (any objective, e.g. a network trained by the
 * caller's framework): the caller has written W_i = X_i - eta * (sum of its H local gradients)
 * into the LIVE matrix (swarm_models_ptr) with work ordered before the handle's stream, and
 * declares those nodes' steps pending; the next round adds W_i - X_i on top of the average
 * exactly as for the built-in objectives.  nodes: host array of `count` distinct ids, or NULL
 * for all nodes.  No objective needs to be set.  SWARM_ESTATE in INPLACE mode (there the caller
 * updates the COMM matrix itself and nothing is pending). */
swarm_status swarm_mark_pending(swarm_t h, const uint32_t *nodes, uint32_t count);

/* Random maximal matching of G for the current round (round model: nodes meet in
 * disjoint pairs).  Edges get random 64-bit priorities; an edge is kept when both
 * endpoints are free, scanning by increasing priority.  pairs_host receives up to
 * floor(n/2) pairs (2 uint32 each) in increasing edge index.  Synchronises. */
swarm_status swarm_sample_matching(swarm_t h, uint32_t *pairs_host, uint32_t *npairs);

/* Draws, for every node, the staleness of its next read: uniform on {0..S}, limited to
 * the number of rounds done.  stale_host: n bytes.  Does not touch the device. */
swarm_status swarm_sample_stale(swarm_t h, uint8_t *stale_host);

/* The numbers of local steps H_i the nodes take for the current round (n bytes): H for every
 * node under SWARM_STEPS_CONSTANT, else this round's geometric draws.  Does not touch the device. */
swarm_status swarm_sample_steps(swarm_t h, uint8_t *steps_host);

/* One gossip round (Section 3 "Parallel Execution"): every node publishes the code of
 * its model X_i into ring slot r mod (S+1); for every pair (i, j), i decodes the code j
 * published stale[i] rounds ago against X_i and sets
 *     X_i <- (Q(X_i) + Q(X_j)) / 2 + (W_i - X_i),
 * and j does the same with roles swapped; unmatched nodes apply their own pending steps
 * (X_u <- W_u).  Clears the pending marks and advances the round counter.
 * pairs_host: npairs disjoint edges of G (2 uint32 each), or NULL to sample the matching
 * internally.  stale_host: n bytes indexed by reading node, or NULL for fresh reads. */
swarm_status swarm_gossip_round(swarm_t h, const uint32_t *pairs_host, uint32_t npairs,
                                const uint8_t *stale_host);

/* The same round in one pass, for objectives whose gradient is per-coordinate (the diagonal
 * quadratic): equivalent, bit for bit, to swarm_local_steps(all nodes) followed by
 * swarm_gossip_round(pairs, stale), but the H local steps of each node are taken in registers
 * inside the gossip pass and the live copies W are neither written nor read (W keeps its old
 * contents).  Needs bits > 0, H > 0, the diagonal objective and no pending local steps
 * (SWARM_ESTATE otherwise). */
swarm_status swarm_round_fused(swarm_t h, const uint32_t *pairs_host, uint32_t npairs,
                               const uint8_t *stale_host);

/* One step of Algorithm 1 (sequential model), initiator i, responder j adjacent to i:
 * i runs its H local steps from its snapshot Xhat_i, then
 *     X_i <- (Q(X_i) + Q(X_j)) / 2 + (W_i - Xhat_i),   X_j <- (Q(X_i) + Q(X_j)) / 2,
 * Xhat_i <- X_i.  Requires stale_max = 0 and DEFERRED apply mode. */
swarm_status swarm_interact(swarm_t h, uint32_t i, uint32_t j);

/* The next `count` steps of Algorithm 1, pairs drawn as by swarm_sample_pair, with the result --
 * models, snapshots, registers, counters -- that `count` calls of swarm_sample_pair + swarm_interact
 * give, bit for bit.  Interactions on disjoint node sets commute (Section 2, "The Distributed System
 * Model": the unit of time is one pairwise interaction, and Theta(n) of them can occur in parallel),
 * so each interaction joins the earliest kernel launch after the last one that touches either of its
 * nodes, and a launch carries all its interactions as grid rows; no per-interaction host work or
 * copy remains.  For the diagonal objective (fixed-width codes) the initiator's local steps are
 * taken inside the interaction kernel and the live copy W is neither written nor read (it keeps its
 * old contents); for the other objectives they are one more launch per group.
 * pairs_host: receives the 2*count node ids (initiator, responder) in the order of Algorithm 1, or
 * NULL.  launches: receives the number of interaction launches, or NULL.  Same requirements as
 * swarm_interact. */
swarm_status swarm_run_sequential(swarm_t h, uint32_t count, uint32_t *pairs_host, uint32_t *launches);

/* Algorithm 1's sampling: initiator uniform over nodes, responder uniform over its
 * neighbours, for the current interaction number.  Does not touch the device. */
swarm_status swarm_sample_pair(swarm_t h, uint32_t *i, uint32_t *j);

/* Stateless codec (Corollary 2.1: Enc, and Dec with a decoding key).
 * quantize: x_dev (d floats) -> codes_dev (d*bits/8 bytes; coordinate k occupies bits
 * [k*bits, (k+1)*bits) of a little-endian bit stream), stochastic rounding drawn from the
 * stream (seed, node, event).  dequantize: out[k] = eps * (member of the code's residue
 * class nearest to key[k]/eps).  d a multiple of 8; bits in {2,4,8,16}. */
swarm_status swarm_quantize(const float *x_dev, uint64_t d, float eps, uint32_t bits,
                            uint64_t seed, uint32_t node, uint32_t event, void *codes_dev,
                            void *hip_stream);
swarm_status swarm_dequantize(const void *codes_dev, const float *key_dev, uint64_t d, float eps,
                              uint32_t bits, float *out_dev, void *hip_stream);

/* Copy columns [k0, k0+len) of nodes [node0, node0+count) between the device matrix
 * `which` (SWARM_MODELS_*) and a host array of count x len floats.  Writing LIVE marks
 * those nodes pending; writing COMM clears the mark.  Synchronise. */
swarm_status swarm_read_models(swarm_t h, uint32_t which, uint32_t node0, uint32_t count,
                               uint64_t k0, uint64_t len, float *dst_host);
swarm_status swarm_write_models(swarm_t h, uint32_t which, uint32_t node0, uint32_t count,
                                uint64_t k0, uint64_t len, const float *src_host);
/* Exact resume.  Every random draw is a function of (seed, round or interaction number, ids), so
 * the model matrices, the registers, the counters, the pending marks and the round counters are the
 * whole state of a run: a handle created with the same configuration and graph that loads the image
 * continues bit for bit as the saved one would have (objective data are borrowed and not part of
 * it: set the objective again).  swarm_state_bytes gives the image size for the handle as it stands;
 * images are host memory; a load into a handle of another configuration is SWARM_EINVAL.
 * All three synchronise. */
swarm_status swarm_state_bytes(swarm_t h, uint64_t *nbytes);
swarm_status swarm_save_state(swarm_t h, void *dst_host, uint64_t nbytes);
swarm_status swarm_load_state(swarm_t h, const void *src_host, uint64_t nbytes);

/* Device address of a model matrix (n x d floats, row-major), for zero-copy views. */
swarm_status swarm_models_ptr(swarm_t h, uint32_t which, float **ptr_dev);

/* Packed codes a node published `age` rounds before the last completed round
 * (age <= S): bytes [byte0, byte0+len) of its code row.  Synchronises. */
swarm_status swarm_read_codes(swarm_t h, uint32_t age, uint32_t node, uint64_t byte0,
                              uint64_t len, uint8_t *dst_host);

/* Reductions.  potential: Gamma = sum_i |X_i - mu|^2 with mu the mean model (Section 4,
 * "Proof Overview"), accumulated in float64; mu_dev (d floats, device) may be NULL.
 * pair_linf: max_k |X_i[k] - X_j[k]| for each given pair (the distance that decides
 * whether decoding succeeds).  Both synchronise. */
swarm_status swarm_potential(swarm_t h, double *gamma_host, float *mu_dev);
swarm_status swarm_pair_linf(swarm_t h, const uint32_t *pairs_host, uint32_t npairs,
                             float *linf_host);

/* The potential for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same reduction as swarm_potential over a
 * caller-owned n x d float32 matrix X_dev (row-major, 16-byte aligned, d a positive multiple of 4),
 * with the per-workgroup partial sums in a fixed 1 MiB device array inside the library instead of a
 * buffer of a handle.  Needs no handle, allocates nothing, does not synchronise: the kernels are
 * enqueued on hip_stream, Gamma arrives in gamma_dev (one double, device) and, if mu_dev is not NULL,
 * the mean model in mu_dev (d floats, device, 16-byte aligned).  d is limited to 134217728 coordinates
 * (SWARM_EINVAL beyond; text from swarm_last_error(NULL)).  Every call on a GPU shares that GPU's
 * array: calls that overlap on one GPU (different streams or threads) race and must be serialised by
 * the caller.  Nothing in the array has to be cleared between calls: a call overwrites every partial
 * sum it later reads. */
swarm_status swarm_potential_static(const float *X_dev, uint32_t n, uint64_t d, double *gamma_dev,
                                    float *mu_dev, void *hip_stream);

/* SWARM_SCALE_GLOBAL_LINF: the scale the next round will use and the largest disagreement
 * max |X_i - decoded partner| of the last round that had pairs (0 before the first).  Other
 * policies: cfg.eps and 0.  Either pointer may be NULL (host memory).  Synchronises. */
swarm_status swarm_scale(swarm_t h, float *eps_next, float *disagreement);

/* SWARM_CODEC_PREFIX: how many tile reads stopped after 4, 8 and 16 bits per coordinate since init
 * (tiles[3], host memory) and how many tiles no level confirmed.  Zeros for the fixed codec.
 * Synchronises. */
swarm_status swarm_prefix_stats(swarm_t h, uint64_t *tiles, uint64_t *unconfirmed);

/* Counters since init.  interactions: pairwise interactions (the paper's unit of time);
 * bits_communicated: bits read from or written to another node's buffer; decode_failures:
 * coordinates where a fresh read decoded to another lattice point than the sender's.
 * Returns SWARM_ERANGE if the clamp was reached since init.  Synchronises. */
swarm_status swarm_counters(swarm_t h, uint64_t *rounds, uint64_t *interactions,
                            uint64_t *bits_communicated, uint64_t *decode_failures);

const char *swarm_last_error(swarm_t h);

#ifdef __cplusplus
}
#endif
#endif /* SWARM_H */
