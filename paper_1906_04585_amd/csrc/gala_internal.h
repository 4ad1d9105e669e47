// Internal declarations shared by the host side and the kernel files of libgala.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>

namespace gala {

// Fixed geometry of the network (App. C.2 of the paper: three convolutions, one hidden
// layer, two linear heads) on 4 x 84 x 84 byte frames.
constexpr int C0 = 4, H0 = 84, W0 = 84, FRAME = C0 * H0 * W0;            // 28224 bytes
constexpr int C1 = 32, H1 = 20, W1 = 20, K1 = 8, S1 = 4, P1 = H1 * W1;    // conv1 out
constexpr int C2 = 64, H2 = 9, W2 = 9, K2 = 4, S2 = 2, P2 = H2 * W2;      // conv2 out
constexpr int C3 = 64, H3 = 7, W3 = 7, K3 = 3, S3 = 1, P3 = H3 * W3;      // conv3 out
constexpr int FLAT = C3 * P3;                                            // 3136
constexpr int FC = 512;
constexpr int A1SZ = P1 * C1, A2SZ = P2 * C2, A3SZ = FLAT;                // floats per frame
constexpr int KW1 = C0 * K1 * K1, KW2 = K2 * K2 * C1, KW3 = K3 * K3 * C2; // 256, 512, 576

// Offsets (in floats) of every tensor inside one agent's slice of a parameter-shaped
// arena (parameters, gradients, RMSprop state and history all use the same map).
// Internal orderings, chosen for the kernels that read them:
//   w1  [k = (c, kh, kw)][o]          256 x 32
//   w2  [k = (kh, kw, c)][o]          512 x 64
//   w3  [k = (kh, kw, c)][o]          576 x 64
//   fcw [j][k = (h, w, c)]            512 x 3136   (activations are channels-last)
//   piw [a][j], vw [j]
struct Layout {
    int n_actions;
    long w1, b1, w2, b2, w3, b3, fcw, fcb, piw, pib, vw, vb;
    long d;       // canonical parameter count
    long d_pad;   // slice stride, multiple of 256 floats; the tail stays zero
};

inline Layout make_layout(int n_actions)
{
    Layout L{};
    L.n_actions = n_actions;
    long off = 0;
    auto take = [&](long n) { long o = off; off += (n + 63) / 64 * 64; return o; };
    L.w1 = take((long)KW1 * C1); L.b1 = take(C1);
    L.w2 = take((long)KW2 * C2); L.b2 = take(C2);
    L.w3 = take((long)KW3 * C3); L.b3 = take(C3);
    L.fcw = take((long)FC * FLAT); L.fcb = take(FC);
    L.piw = take((long)n_actions * FC); L.pib = take(n_actions);
    L.vw = take(FC); L.vb = take(1);
    L.d_pad = (off + 255) / 256 * 256;
    L.d = (long)KW1 * C1 + C1 + (long)KW2 * C2 + C2 + (long)KW3 * C3 + C3 + (long)FC * FLAT + FC +
          (long)n_actions * FC + n_actions + FC + 1;
    return L;
}

// One tensor of the canonical parameter vector viewed as a 4-d row-major array, with
// the strides of the same element inside the internal slice.
struct Segment {
    long canon_off, intern_off;
    int dim[4];
    long stride[4];
    long count;
};
constexpr int N_SEGMENTS = 12;
struct SegmentTable { Segment s[N_SEGMENTS]; };
SegmentTable make_segments(const Layout &L);

struct HParams {
    int T, B;
    float gamma, vf_coef, ent_coef, lr, rms_alpha, rms_eps, max_grad_norm;
    int compute_dtype;           // 0 = fp32 MFMA, 1 = bf16 MFMA with fp32 master weights and accumulation
};

// Device buffers of one context.  M = T*B rollout frames, F = M + B frames incl. bootstrap.
struct Buffers {
    float *x[2];      // [N][d_pad] parameters, ping-pong for the mixing step
    float *g;         // [N][d_pad] gradients
    float *v;         // [N][d_pad] RMSprop second moments
    float *hist;      // [tau+1][N][d_pad] broadcast history (tau > 0 only)
    float *a1, *a2, *a3, *h;          // [N][F][..] activations, channels-last
    float *logits, *values;           // [N][M][A], [N][F]
    float *ret, *adv;                 // [N][M]
    float *dlogits, *dvalues;         // [N][M][A], [N][M]
    float *loss_part;                 // [N][M][3]: per-sample policy term, squared value error, entropy
    float *dzh, *dz3, *dz2, *dz1;     // [N][M][..] pre-activation gradients
    float *ws;                        // split-K partial sums
    float *norm_part;                 // [N][NORM_PARTS]
    float *gbar, *gbar_part;          // [d_pad] gradient averaged over agents, [grad_mean_blocks] its squares
    float *gram_part, *gram, *cosm;   // [pairs][chunks][GRAM_T^2] partial Gram tiles, [N][N] Gram, [N][N] cosine
    float *upd_part, *upd_norm;       // [N][UPDATE_NORM_BLOCKS], [N] row norms + [2] (largest row, Frobenius)
    float *stats;                     // [N][5]
    float *cons_part;                 // [N][4 * consensus_blocks] partial sums of squares + 2 results
    float *row_ss;                    // [N] scratch of the norm reductions
    int32_t *peer, *delay;            // [phases][N][max_in]
    int32_t *cyc_order, *cyc_start;   // [phases][N], [phases][N + 1]: the peer permutation's cycles (if it is one)
    float *weight;                    // [phases][N][max_in+1]
};

// Per-agent partial sums of squared gradients written by the kernels that produce the gradient:
// one per output tile of the hidden layer's weight gradient, then one per workgroup of the
// convolutions' split reductions.  NORM_USED of the NORM_PARTS entries of a row are in use.
constexpr int NORM_PARTS = 256;
constexpr int FC_WGRAD_TILES = 100;
constexpr int NORM_USED = 179;
// Activation and gradient buffers (a1, a2, a3, h, dz1..dz3, dzh) are allocated with this many
// zero floats in front of the data.  Kernels that must treat a group as zero (a padding tap
// of a transposed convolution, the tail of a k-range) read it from there instead of masking.
constexpr int ZERO_PAGE = 64;

// Optional per-phase timing with HIP events on the context's stream (diagnostic).
struct PhaseTimer {
    bool on = false;
    hipStream_t stream = nullptr;
    std::vector<hipEvent_t> ev;
    std::vector<const char *> names;
    int n = 0;
    void begin() { n = 0; mark("start"); }
    void mark(const char *name)
    {
        if (!on) return;
        if (n >= (int)ev.size()) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return;
            ev.push_back(e);
            names.push_back(name);
        }
        names[n] = name;
        (void)hipEventRecord(ev[n], stream);
        ++n;
    }
};

// ---- launchers (each enqueues on `s` and returns hipGetLastError()) ---------------------
struct NetArgs {
    int N, M, F, Bn;              // agents, rollout frames, all frames, bootstrap frames
    Layout L;
    const float *x;              // current parameters
    Buffers b;
    const uint8_t *obs, *boot;
    bool bf16;                   // conv/fc operands rounded to bf16 in LDS, fp32 accumulation
};

// before_fc: an event the stream waits for in front of the hidden layer (the first kernel that reads the
// hidden layer's weights), or nullptr
hipError_t launch_forward(const NetArgs &a, hipStream_t s, PhaseTimer *pt, hipEvent_t before_fc = nullptr);
// returns, advantages, loss terms per sample, head output gradients and the hidden layer's dzh
hipError_t launch_loss(const NetArgs &a, const HParams &hp, const int32_t *actions, const float *rewards,
                       const uint8_t *dones, hipStream_t s);
// number of entries of actions[0..n) outside [0, A), written to *count (one workgroup, no atomics)
hipError_t launch_count_bad_actions(const int32_t *actions, long n, int A, int32_t *count, hipStream_t s);
hipError_t launch_sample(int N, int Bn, int A, const float *logits, const float *values, uint64_t seed, long step,
                         int32_t *actions, float *values_out, float *logp_out, hipStream_t s);
// Second stream (default priority) and the events that order it against the context's stream.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork[4] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t join = nullptr;
    hipEvent_t opt_fork = nullptr, opt_done = nullptr;   // the hidden layer's share of the optimizer pass (optional overlap)
};
// data gradients and conv1's weight gradient on `s`, the other weight gradients on the side stream; ends with every
// agent's loss terms, gradient norm and clip factor in stats
hipError_t launch_backward(const NetArgs &a, const HParams &hp, hipStream_t s, PhaseTimer *pt, const SideStream *side);
size_t workspace_floats(int N, int M, int F);

hipError_t launch_rmsprop(int N, const Layout &L, const HParams &hp, float *x, float *v, const float *g,
                          bool shared_gradient, const float *stats, hipStream_t s);
int grad_mean_blocks(const Layout &L);
hipError_t launch_grad_mean(int N, const Layout &L, const HParams &hp, const float *g, float *gbar, float *part,
                            float *stats, hipStream_t s);
bool fused_mix_available(int N);
hipError_t launch_rmsprop_mix_cycles(int N, const Layout &L, const HParams &hp, float *x, float *v, const float *g,
                                     const int32_t *order, const int32_t *cstart, int n_cycles, const float *weight,
                                     const float *stats, hipStream_t s, long col_begin = 0, long col_end = -1);
hipError_t launch_rmsprop_mix(int N, const Layout &L, const HParams &hp, float *x, float *v, const float *g,
                              float *hist, int tau, long round, int phase, int max_in, const int32_t *peer,
                              const int32_t *delay, const float *weight, const float *stats, hipStream_t s);
hipError_t launch_publish(int N, const Layout &L, const float *x, float *hist_slot, hipStream_t s);
hipError_t launch_mix(int N, const Layout &L, const float *x_in, float *x_out, const float *hist, int tau,
                      long round, int phase, int max_in, const int32_t *peer, const int32_t *delay,
                      const float *weight, hipStream_t s);
// diagnostics (Sec. 5 "Effects of gossip")
constexpr int GRAM_T = 32;                 // agents per tile side of the gradient Gram matrix
constexpr int UPDATE_NORM_BLOCKS = 64;
int gram_pairs(int N);
int gram_chunks(int N);
hipError_t launch_grad_cosine(int N, const Layout &L, const float *g, float *part, float *gram, float *cosm,
                              hipStream_t s);
hipError_t launch_update_norm(int N, const Layout &L, const HParams &hp, const float *g, bool shared_gradient,
                              const float *v, const float *stats, float *part, float *row_ss, float *out,
                              hipStream_t s);
// Consensus distance.  Up to CONS_REG_AGENTS agents: at most CONS_BLOCKS workgroups of four
// wavefronts, one partial sum of squares per (agent, wavefront); more agents: one partial per
// (agent, 1024 columns).  consensus_parts gives the partials per agent for sizing the scratch buffer.
constexpr int CONS_BLOCKS = 512;
constexpr int CONS_REG_AGENTS = 64;
int consensus_parts(int N, const Layout &L);
hipError_t launch_row_norms(const float *part, int rows, int cols, float *row_ss, float *row_norm, float *result,
                            hipStream_t s);
hipError_t launch_consensus(int N, const Layout &L, const float *x, float *part, float *row_ss, float *result,
                            hipStream_t s);
hipError_t launch_permute(int N, const Layout &L, const SegmentTable &tab, float *canon, float *intern,
                          int to_internal, hipStream_t s);

}  // namespace gala
