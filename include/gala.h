/*
 * gala.h -- C ABI of the MI355X (gfx950) GALA-A2C hot path.
 *
 * One context holds N independent A2C actor-learners that share one GPU
 * (Sec. 3 of "Gossip-based Actor-Learner Architectures for Deep Reinforcement
 * Learning").  A training round is Algorithm 1 for all agents at once:
 *     gala_learner_step   returns/advantages + one A2C optimisation step per agent
 *     gala_gossip         broadcast + parameter averaging over the peer topology
 * Every step of both calls runs in HIP kernels on the stream given at creation.
 *
 * Conventions
 *   - "dev" pointers are device memory on the GPU that was current when the
 *     context was created; "host" pointers are ordinary host memory.
 *   - Input buffers are borrowed: the caller keeps them alive and unmodified until
 *     the work enqueued by the call has completed on the context's stream.
 *     gala_learner_step and gala_gossip only enqueue; they never synchronise.
 *     Calls that copy to a host pointer synchronise the stream before returning.
 *   - All memory the library needs is allocated in gala_create and released in
 *     gala_destroy; the hot calls allocate nothing.
 *   - Every function returns 0 on success or a negative GALA_E* code;
 *     gala_last_error() gives a text for the most recent failure of a context
 *     (or of gala_create when passed NULL).  No exceptions cross this boundary.
 *   - Parameter vectors use the canonical per-agent order
 *         conv1.w conv1.b conv2.w conv2.b conv3.w conv3.b fc.w fc.b pi.w pi.b v.w v.b
 *     with convolution weights OIHW row-major, dense weights (out, in) row-major and
 *     the hidden layer's inputs ordered channel, row, column.  [N][d] means agent-major.
 *     The library keeps its own internal ordering; get/set convert.
 */
#ifndef GALA_H
#define GALA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GALA_OK       0
#define GALA_EINVAL  -1   /* bad argument, unsupported shape, invalid topology      */
#define GALA_ENOMEM  -2   /* device or host allocation failed                       */
#define GALA_EHIP    -3   /* a HIP runtime call failed (text in gala_last_error)    */
#define GALA_ESTATE  -4   /* call order violated (e.g. gossip round went backwards) */

typedef struct gala_ctx gala_ctx;   /* opaque, owned by the library */

/* The network of App. C.2: three unpadded convolutions with ReLU (8x8 stride 4,
 * 4x4 stride 2, 3x3 stride 1), one hidden layer with ReLU, a linear policy head and
 * a linear value head.  Kernel sizes and strides are fixed; this build accepts
 * in_c=4, in_h=in_w=84, c1=32, c2=64, c3=64, fc=512 and 1 <= n_actions <= 64. */
typedef struct {
    int in_c, in_h, in_w;
    int c1, c2, c3;
    int fc;
    int n_actions;
} gala_net_dims;

/* Table 2 of the paper plus the rollout shape.  T = horizon N (5), B = simulators
 * per learner (16).  RMSprop: v <- rms_alpha v + (1-rms_alpha) g^2,
 * x <- x - lr g / (sqrt(v) + rms_eps), momentum 0.  Gradients are rescaled per
 * agent by min(1, max_grad_norm / (||g||_2 + 1e-6)) first. */
typedef struct {
    int   T, B;
    float gamma, vf_coef, ent_coef;
    float lr, rms_alpha, rms_eps;
    float max_grad_norm;
    int   compute_dtype;       /* 0 = fp32 matrix instructions; 1 = conv/fc operands rounded to bf16
                                  (fp32 parameters, activations and accumulation; everything else fp32) */
} gala_hparams;

#define GALA_TOPO_RING      0   /* directed ring v1->v2->...->vn->v1: agent i receives from i-1 (Fig. 5) */
#define GALA_TOPO_EXP       1   /* 1-peer exponential graph: at round r agent i mixes with
                                   (i + 2^(r mod log2 N)) mod N; N must be a power of two       */
#define GALA_TOPO_EXPLICIT  2   /* caller-supplied peers and weights, n_phases tables cycled by round */
#define GALA_TOPO_EXP_REVERSE 3 /* the exponential graph with every edge turned round: agent i mixes with
                                   (i - 2^(r mod log2 N)) mod N.  Both directions give the doubly
                                   stochastic P = (I + shift)/2 of Sec. 2; N a power of two          */

/* Mixing weights follow Algorithm 1: 1/(1+|N_in|) for ring and exponential graphs.
 * max_delay = tau bounds message staleness; each edge (phase, receiver[, in-peer slot])
 * gets a fixed delay splitmix64(delay_seed + edge_index) mod (tau+1) rounds, where
 * edge_index = (phase * N + receiver) * max_in + slot.  An agent whose delayed message
 * was never sent (round - delay < 0) skips averaging that round.
 * For GALA_TOPO_EXPLICIT: peers is host int32 [n_phases][N][max_in] (-1 = unused slot),
 * weights is host float [n_phases][N][max_in+1] with the self weight first; rows must be
 * non-negative and sum to 1 within 1e-5 (row-stochastic, Sec. 2). */
typedef struct {
    int            kind;
    int            max_delay;
    uint64_t       delay_seed;
    const int32_t *peers;
    const float   *weights;
    int            n_phases;
    int            max_in;
} gala_topology;

/* Create a context for n_agents agents.  hip_stream is a hipStream_t (NULL = the
 * default stream) on which all work is enqueued.  Parameters start at zero and the
 * RMSprop state at zero; call gala_set_params before the first learner step (a learner,
 * round, comparator or acting step before it fails with GALA_ESTATE).
 * Limits: 1 <= n_agents <= 4096, T*B <= 4096 and n_agents * (T*B + B) <= 83 886 frames per
 * context (the kernels address an agent's activations with 32-bit byte offsets); beyond
 * them the call fails with GALA_EINVAL.
 * If the environment variable GALA_CHECK_ACTIONS is set when the context is created, every
 * learner, round and comparator step first counts the actions outside [0, n_actions) with
 * a small kernel, waits for the count and fails with GALA_EINVAL when it is not zero (a
 * debugging aid: it synchronises the stream on every step).
 * The context also owns one internal stream of default priority on which the weight-gradient
 * kernels of a learner step run beside the data-gradient chain; it is forked from and joined
 * back into hip_stream inside every call, so callers only ever order against hip_stream.
 * Setting the environment variable GALA_SINGLE_STREAM before gala_create keeps everything on
 * hip_stream (same kernels, same results).
 * Setting GALA_OVERLAP_OPTIMIZER before gala_create makes gala_round (one in-peer, no delays) run the
 * hidden layer's share of its optimizer + mixing pass on the internal stream, beside the convolutions
 * of the next gala_round's forward pass, which waits for it in front of the hidden layer; every other
 * entry point waits for it first.  Same kernels on the same values: identical results.  Measured no
 * faster on one device (the pass and the byte-reading convolution compete for memory), hence opt-in. */
int gala_create(gala_ctx **out, int n_agents, const gala_topology *topo,
                const gala_net_dims *net, const gala_hparams *hp, void *hip_stream);
int gala_destroy(gala_ctx *ctx);

/* Parameters per agent (d), for sizing [N][d] buffers. */
size_t gala_param_count(const gala_ctx *ctx);
const char *gala_last_error(const gala_ctx *ctx);

/* [N][d] float, canonical order; is_device says whether the pointer is dev or host. */
int gala_set_params(gala_ctx *ctx, const float *src, int src_is_device);
int gala_get_params(gala_ctx *ctx, float *dst, int dst_is_device);
/* RMSprop second-moment estimates v, same shape and order. */
int gala_set_opt_state(gala_ctx *ctx, const float *src, int src_is_device);
int gala_get_opt_state(gala_ctx *ctx, float *dst, int dst_is_device);

/* One A2C learner step for every agent (Algorithm 1: compute returns and advantages,
 * then one optimisation step on the TD loss Eq. (1) and the batched policy gradient with
 * entropy Eq. (4)).  All pointers dev:
 *   obs_u8        uint8 [N][T][B][4][84][84]  states s_t (scaled by 1/255 inside)
 *   actions       int32 [N][T][B]             in [0, n_actions); out-of-range is undefined
 *                                             unless GALA_CHECK_ACTIONS is set (see gala_create)
 *   rewards       float [N][T][B]
 *   dones         uint8 [N][T][B]             1 = the transition at t ended the episode
 *   bootstrap_obs uint8 [N][B][4][84][84]     state reached after the last action */
int gala_learner_step(gala_ctx *ctx, const uint8_t *obs_u8, const int32_t *actions,
                      const float *rewards, const uint8_t *dones, const uint8_t *bootstrap_obs);

/* One gossip iteration x_i <- sum_j p_ij x_j over the topology's table for this round
 * (Sec. 2 "Gossip algorithms"; Algorithm 1, broadcast + averaging; Eq. (6) with delays).
 * Rounds must be passed in increasing order starting at 0 when max_delay > 0. */
int gala_gossip(gala_ctx *ctx, int64_t round);

/* One whole round of Algorithm 1 (optimise, broadcast, average) in a single call: the same
 * result, bit for bit, as gala_learner_step followed by gala_gossip(round), same arguments
 * and rules, but clipping, RMSprop and the mixing step run as one kernel, so parameters,
 * gradients and optimizer state cross HBM once (20 bytes per parameter instead of 32).
 * Topologies with one in-peer per agent and no delays whose peers form a permutation (ring,
 * exponential graph, explicit permutations) are walked cycle by cycle, any number of agents;
 * otherwise a workgroup owns a block of parameter columns of all agents and keeps their
 * updated values in LDS, and for more than 256 agents the call runs the two separate steps. */
int gala_round(gala_ctx *ctx, const uint8_t *obs_u8, const int32_t *actions, const float *rewards,
               const uint8_t *dones, const uint8_t *bootstrap_obs, int64_t round);

/* Synchronous A2C with gradient averaging, the method GALA-A2C is compared with (Sec. 5,
 * "Experimental setup": every agent averages its gradient with all others before each
 * update, which for identical replicas is the batched update of Eq. (5) over all agents'
 * simulators).  Same inputs as gala_learner_step.  Every agent's gradient is computed at its
 * own parameters; gbar = (1/N) sum_i g_i (agents added in index order) is clipped once by its
 * own global norm and applied by every agent with RMSprop to its own parameters and state.
 * No gossip follows.  Afterwards gala_get_grads returns the agents' own gradients,
 * gala_get_mean_grad returns gbar, and the norm / clip columns of gala_get_step_stats hold
 * gbar's values in every row. */
int gala_a2c_allreduce_step(gala_ctx *ctx, const uint8_t *obs_u8, const int32_t *actions,
                            const float *rewards, const uint8_t *dones, const uint8_t *bootstrap_obs);
/* Pre-clip average gradient of the last gala_a2c_allreduce_step, [d] float canonical. */
int gala_get_mean_grad(gala_ctx *ctx, float *dst, int dst_is_device);

/* Acting step of Algorithm 1 ("take actions according to pi") for every agent's B simulators:
 * a forward pass of the current parameters over one state per simulator, then one draw per
 * state from pi = softmax(logits).  All pointers dev:
 *   obs_u8  uint8 [N][B][4][84][84]   current states
 *   actions int32 [N][B]              out: sampled actions
 *   values  float [N][B]              out: V(s) (may be NULL)
 *   logp    float [N][B]              out: log pi(a|s) of the sampled action (may be NULL)
 * The draw inverts the distribution function: with u = (top 24 bits of
 * splitmix64(seed + counter)) / 2^24, counter = (step * N + agent) * B + simulator, the action is
 * the first one whose running sum pi_0 + ... + pi_a exceeds u.  The same (seed, step) always
 * gives the same actions.  The call reuses the activation buffers of the learner step: the
 * outputs and activations of the previous gala_learner_step are no longer readable afterwards. */
int gala_act(gala_ctx *ctx, const uint8_t *obs_u8, uint64_t seed, int64_t step, int32_t *actions,
             float *values, float *logp);

/* ---- diagnostics used by tests and logging -------------------------------------- */

/* Pre-clip gradients of the last learner step, [N][d] canonical. */
int gala_get_grads(gala_ctx *ctx, float *dst, int dst_is_device);
/* host float [N][5]: policy-gradient term, TD term, entropy, pre-clip gradient norm,
 * clip factor of the last learner step. */
int gala_get_step_stats(gala_ctx *ctx, float *dst_host);
/* Network outputs of the last learner step, host buffers (any may be NULL):
 * logits [N][T*B][A], values [N][T*B+B] (rollout states, then bootstrap states),
 * returns and advantages [N][T*B]. */
int gala_get_outputs(gala_ctx *ctx, float *logits, float *values, float *returns, float *advantages);
/* Distance from consensus (Prop. 1): max_i ||x_i - mean||_2 and ||X - mean||_F, host floats. */
int gala_consensus_distance(gala_ctx *ctx, float *max_dist, float *frob);
/* The same quantities for callers that cannot allocate device memory or wait for the stream (code
 * under HIP graph capture, tight serving or logging loops, harnesses that forbid hipMalloc): the same
 * kernels as gala_consensus_distance, enqueued on the context's stream with no allocation and no
 * synchronisation.  result_dev is a dev float[2] that receives max_i ||x_i - mean||_2 and ||X - mean||_F
 * once the enqueued work has run.  The partial sums live in a 1 MiB array that is part of the library
 * image (one copy per GPU, held until the process ends) instead of the context's own buffer: it holds
 * 262 144 floats, a context needs n_agents * (partials per agent + 1) of them (about 1 650 partials per
 * agent for this network, so up to 158 agents), and a context that needs more is refused with
 * GALA_EINVAL.  All contexts on
 * a GPU share that array, so calls of this function that overlap in time on one GPU (different
 * streams) race; calls on one stream, or otherwise ordered, are safe.  Nothing in the array has to
 * start at zero: every entry that is read was written by the same call. */
int gala_consensus_distance_noalloc(gala_ctx *ctx, float *result_dev);
/* Pair-wise cosine similarity of the agents' gradients of the last learner step (Fig. 2b):
 * cos[i][j] = <g_i, g_j> / (||g_i|| ||g_j||), pre-clip gradients, host float [N][N]; rows and
 * columns of an agent whose gradient is zero are 0.  One pass over the gradient arena. */
int gala_grad_cosine(gala_ctx *ctx, float *cos_host);
/* Size of the last optimiser step in the notation of Prop. 1: row i of the update matrix
 * alpha G is x_i before the step minus x_i after it (before mixing).  row_norms_host: float [N]
 * = ||alpha g_i||_2 (may be NULL); *frob_host = ||alpha G||_F.  Valid after gala_learner_step,
 * gala_round or gala_a2c_allreduce_step and before the next of them. */
int gala_update_norm(gala_ctx *ctx, float *row_norms_host, float *frob_host);
/* Right-hand side of Prop. 1 for agents that started from identical parameters:
 * *bound = sum_{s=0..n-1} beta^(n-s) update_norms[s], where update_norms[s] = ||alpha G^(s)||
 * of round s (gala_update_norm) and beta in [0, 1] is the contraction factor of the mixing
 * matrices (cos(pi/N) for the directed ring with weights 1/2).  Host arithmetic only. */
int gala_prop1_bound(double beta, const double *update_norms, int n, double *bound);
/* Output gradients of the two heads as the loss kernel of the last learner step wrote them, host
 * buffers (either may be NULL): dlogits [N][T*B][A] = dLoss/dlogits, dvalues [N][T*B] = dLoss/dV.
 * With the entropy coefficient at zero a row of dlogits is A_m (pi - onehot(a_m)) / (T*B): the
 * taken action is the one entry whose sign differs, which lets a test check the integer gather. */
int gala_get_head_grads(gala_ctx *ctx, float *dlogits_host, float *dvalues_host);
/* In-peer and delay tables the library will use at `round`, host int32 [N][max_in] each
 * (max_in = 1 for ring and exponential graphs). */
int gala_get_peer_table(gala_ctx *ctx, int64_t round, int32_t *peer, int32_t *delay);

/* Activations of the last learner step, host float, channels-last as the kernels keep
 * them: layer 1 -> [N][F][20][20][32], 2 -> [N][F][9][9][64], 3 -> [N][F][7][7][64],
 * 4 -> hidden [N][F][512]; F = T*B + B frames (rollout states, then bootstrap states),
 * values after ReLU. */
int gala_get_activations(gala_ctx *ctx, int layer, float *dst_host);

/* Per-phase timing (diagnostic).  While enabled, gala_learner_step and gala_gossip record a
 * HIP event on the context's stream after every phase (conv1_fwd, ..., clip_rmsprop,
 * gossip_mix).  gala_get_phase_times synchronises and returns the elapsed milliseconds
 * between consecutive events recorded since the last learner step began: names receives
 * the phase names joined by ';' (host, names_cap bytes), ms the durations (host, cap
 * floats), *n_out how many. */
int gala_set_profiling(gala_ctx *ctx, int enabled);
int gala_get_phase_times(gala_ctx *ctx, char *names, size_t names_cap, float *ms, int cap, int *n_out);

#ifdef __cplusplus
}
#endif
#endif /* GALA_H */
