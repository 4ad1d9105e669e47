// Returns/advantages and the A2C loss with its head gradients (wavefront reductions),
// per-agent global-norm clipping fused with RMSprop, the gossip mixing pass, the
// distance-from-consensus reduction, and the canonical <-> internal parameter permutation.
#include "gala_internal.h"

namespace gala {

static __device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Block-wide sum over 256 threads (4 wavefronts), result valid in every thread.
static __device__ __forceinline__ float block_sum_256(float v, float *red)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// ---- Algorithm 1, "compute returns and advantages" + loss of Eq. (1) and Eq. (4), and the gradient
// that the two heads send back into the hidden layer -------------------------------------------------
//   G_t = r_t + gamma (1 - done_t) G_{t+1},  G_T = V(state after the last action);  A_t = G_t - V_t
//   loss = mean(-log pi(a_t|s_t) A_t) + c_v mean((G_t - V_t)^2) - eta mean(H_t),  G and A constants
//   dloss/dz_k = [A (pi_k - 1[k = a]) + eta pi_k (log pi_k + H)] / M,   dloss/dV = -2 c_v (G - V) / M
//   (pi_a - 1 is formed as -sum_{k != a} pi_k)
//   dzh[f][j] = (sum_a W_pi[a][j] dlogits[f][a] + w_v[j] dvalue[f]) * (h[f][j] > 0)
// One workgroup per (LOSS_FRAMES samples, agent), one wavefront per sample and one lane per action
// for the loss part: every wavefront walks its simulator's rollout back from the last step to its
// own (at most T steps) instead of waiting for a pass over the whole rollout.  The per-sample loss
// terms go to loss_part[agent][sample][3]; the kernel that ends the backward pass sums them in sample order.
// Then a thread owns one hidden column j, reads each head weight once and applies it to all
// LOSS_FRAMES samples, whose output gradients sit in LDS.
constexpr int MAX_ACTIONS = 64;
constexpr int LOSS_FRAMES = 8;
constexpr int LOSS_THREADS = 64 * LOSS_FRAMES;
static_assert(LOSS_THREADS == FC, "one thread per hidden column");

__global__ __launch_bounds__(LOSS_THREADS) void loss_heads_kernel(
    int T, int Bn, float gamma, float vf_coef, float ent_coef, Layout L, const float *__restrict__ logits,
    const float *__restrict__ values, const int32_t *__restrict__ actions, const float *__restrict__ rewards,
    const uint8_t *__restrict__ dones, const float *__restrict__ h, const float *__restrict__ x, float *ret,
    float *adv, float *dlogits, float *dvalues, float *loss_part, float *dzh)
{
    __shared__ float dl[LOSS_FRAMES][MAX_ACTIONS + 1];   // [sample][action], value gradient in slot A
    const int A = L.n_actions;
    const int agent = blockIdx.y, f0 = blockIdx.x * LOSS_FRAMES;
    const int M = T * Bn, F = M + Bn;
    const float *V = values + (long)agent * F;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = f0 + wave;
    const float inv_m = 1.0f / (float)M;
    if (m < M) {
        const int b = m % Bn, t = m / Bn;
        float G = V[M + b];
#pragma unroll 4
        for (int tt = T - 1; tt >= t; --tt) {
            const long i = (long)agent * M + tt * Bn + b;
            const float keep = dones[i] ? 0.f : 1.f;
            G = rewards[i] + gamma * keep * G;
        }
        const float Vm = V[m], Am = G - Vm;
        const bool on = lane < A;
        const float z = on ? logits[((long)agent * M + m) * A + lane] : -INFINITY;
        float zmax = z;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, off, 64));
        // log-sum-exp as zmax + log1p(sum over the other actions): stays accurate when one action
        // dominates (a nearly deterministic policy), where log(1 + tiny) would lose the tiny part
        const int top = __ffsll(__ballot(on && z == zmax)) - 1;
        const float others = wave_sum((on && lane != top) ? expf(z - zmax) : 0.f);
        const float lp = z - (zmax + log1pf(others));
        const float p = on ? expf(lp) : 0.f;
        const float H = -wave_sum(on ? p * lp : 0.f);
        const int act = actions[(long)agent * M + m];      // integer gather of the taken action
        const float lp_act = __shfl(lp, act, 64);
        // pi_a - 1 for the taken action as minus the sum of the other probabilities (no cancellation)
        const float not_act = wave_sum((on && lane != act) ? p : 0.f);
        if (on) {
            const float d = (Am * (lane == act ? -not_act : p) + ent_coef * p * (lp + H)) * inv_m;
            dlogits[((long)agent * M + m) * A + lane] = d;
            dl[wave][lane] = d;
        }
        if (lane == 0) {
            const float dv = -2.f * vf_coef * (G - Vm) * inv_m;
            dvalues[(long)agent * M + m] = dv;
            dl[wave][A] = dv;
            ret[(long)agent * M + m] = G;
            adv[(long)agent * M + m] = Am;
            float *lp3 = loss_part + ((long)agent * M + m) * 3;
            lp3[0] = -lp_act * Am; lp3[1] = (G - Vm) * (G - Vm); lp3[2] = H;
        }
    } else if (lane <= A) {
        dl[wave][lane] = 0.f;
    }
    __syncthreads();
    const float *xa = x + agent * L.d_pad;
    const int j = threadIdx.x;
    float acc[LOSS_FRAMES];
    const float wv = xa[L.vw + j];
#pragma unroll
    for (int fi = 0; fi < LOSS_FRAMES; ++fi) acc[fi] = wv * dl[fi][A];
    // six policy rows are requested at a time (the last one again where fewer remain) and applied in
    // order: one wait for memory per six actions instead of one per action
    for (int a0 = 0; a0 < A; a0 += 6) {
        float w[6];
#pragma unroll
        for (int u = 0; u < 6; ++u) w[u] = xa[L.piw + (long)min(a0 + u, A - 1) * FC + j];
#pragma unroll
        for (int u = 0; u < 6; ++u)
            if (a0 + u < A) {
#pragma unroll
                for (int fi = 0; fi < LOSS_FRAMES; ++fi) acc[fi] += w[u] * dl[fi][a0 + u];
            }
    }
#pragma unroll
    for (int fi = 0; fi < LOSS_FRAMES; ++fi) {
        const int f = f0 + fi;
        if (f < M) dzh[((long)agent * M + f) * FC + j] = h[((long)agent * F + f) * FC + j] > 0.f ? acc[fi] : 0.f;
    }
}

// Opt-in validation of the action buffer: one workgroup counts the entries outside [0, A).
__global__ __launch_bounds__(1024) void count_bad_actions_kernel(const int32_t *__restrict__ actions, long n, int A,
                                                                 int32_t *count)
{
    __shared__ int red[16];
    int bad = 0;
    for (long i = threadIdx.x; i < n; i += 1024) bad += (actions[i] < 0 || actions[i] >= A) ? 1 : 0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_xor(bad, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = bad;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int w = 0; w < 16; ++w) t += red[w];
        *count = t;
    }
}

hipError_t launch_count_bad_actions(const int32_t *actions, long n, int A, int32_t *count, hipStream_t s)
{
    hipLaunchKernelGGL(count_bad_actions_kernel, dim3(1), dim3(1024), 0, s, actions, n, A, count);
    return hipGetLastError();
}

hipError_t launch_loss(const NetArgs &a, const HParams &hp, const int32_t *actions, const float *rewards,
                       const uint8_t *dones, hipStream_t s)
{
    hipLaunchKernelGGL(loss_heads_kernel, dim3((a.M + LOSS_FRAMES - 1) / LOSS_FRAMES, a.N), dim3(LOSS_THREADS), 0, s,
                       hp.T, hp.B, hp.gamma, hp.vf_coef, hp.ent_coef, a.L, a.b.logits, a.b.values, actions, rewards,
                       dones, a.b.h, a.x, a.b.ret, a.b.adv, a.b.dlogits, a.b.dvalues, a.b.loss_part, a.b.dzh);
    return hipGetLastError();
}

// ---- acting (Algorithm 1: take actions according to pi) ------------------------------------------------
// One wavefront per (agent, simulator), one lane per action.  u = top 24 bits of
// splitmix64(seed + counter) / 2^24 with counter = (step * N + agent) * B + simulator; the action is
// the first one whose running sum of exp(z - max z) exceeds u times the total.
static __device__ __forceinline__ uint64_t splitmix64_dev(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void sample_kernel(int N, int Bn, int A, const float *__restrict__ logits,
                                                     const float *__restrict__ values, uint64_t seed, long step,
                                                     int32_t *actions, float *values_out, float *logp_out)
{
    const int lane = threadIdx.x & 63;
    const int s = blockIdx.x * 4 + (threadIdx.x >> 6);          // uniform per wavefront
    if (s >= N * Bn) return;
    const bool on = lane < A;
    const float z = on ? logits[(long)s * A + lane] : -INFINITY;
    float zmax = z;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, off, 64));
    float c = on ? expf(z - zmax) : 0.f;                        // becomes the inclusive running sum
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float t = __shfl_up(c, off, 64);
        if (lane >= off) c += t;
    }
    const float total = __shfl(c, 63, 64);
    const float u = (float)(splitmix64_dev(seed + (uint64_t)((long)step * N * Bn + s)) >> 40) * (1.0f / 16777216.0f);
    const unsigned long long above = __ballot(on && c > u * total);
    const int a = above ? __ffsll(above) - 1 : A - 1;
    const float lp = __shfl(z, a, 64) - (zmax + logf(total));
    if (lane == 0) {
        actions[s] = a;
        if (values_out) values_out[s] = values[s];
        if (logp_out) logp_out[s] = lp;
    }
}

hipError_t launch_sample(int N, int Bn, int A, const float *logits, const float *values, uint64_t seed, long step,
                         int32_t *actions, float *values_out, float *logp_out, hipStream_t s)
{
    hipLaunchKernelGGL(sample_kernel, dim3((N * Bn + 3) / 4), dim3(256), 0, s, N, Bn, A, logits, values, seed, step,
                       actions, values_out, logp_out);
    return hipGetLastError();
}

// ---- clip + RMSprop (Table 2; momentum 0) ---------------------------------------------------------------
// The gradient and the second-moment estimate are touched once per round, hundreds of MB apart
// in time: their loads and stores carry the non-temporal hint so that they stream past the
// caches instead of evicting the parameters and activations that are reused.
typedef float stream_vec4 __attribute__((ext_vector_type(4)));
static __device__ __forceinline__ float4 stream_load4(const float *base, long idx4)
{
    const stream_vec4 t = __builtin_nontemporal_load(reinterpret_cast<const stream_vec4 *>(base) + idx4);
    return make_float4(t.x, t.y, t.z, t.w);
}
static __device__ __forceinline__ void stream_store4(float *base, long idx4, float4 val)
{
    stream_vec4 t; t.x = val.x; t.y = val.y; t.z = val.z; t.w = val.w;
    __builtin_nontemporal_store(t, reinterpret_cast<stream_vec4 *>(base) + idx4);
}

//   g <- c g;  v <- a v + (1 - a) g^2;  x <- x - lr g / (sqrt(v) + eps)
static __device__ __forceinline__ void rmsprop1(float &x, float &v, float g, float c, float lr, float alpha, float om,
                                                float eps)
{
    // explicit roundings: the separate and the fused optimizer passes must agree to the last bit
    g = __fmul_rn(g, c);
    v = __fmaf_rn(alpha, v, __fmul_rn(__fmul_rn(om, g), g));
    x = __fsub_rn(x, __fdiv_rn(__fmul_rn(lr, g), __fadd_rn(sqrtf(v), eps)));
}
static __device__ __forceinline__ void rmsprop4(float4 &xx, float4 &vv, float4 gg, float c, float lr, float alpha,
                                                float om, float eps)
{
    rmsprop1(xx.x, vv.x, gg.x, c, lr, alpha, om, eps); rmsprop1(xx.y, vv.y, gg.y, c, lr, alpha, om, eps);
    rmsprop1(xx.z, vv.z, gg.z, c, lr, alpha, om, eps); rmsprop1(xx.w, vv.w, gg.w, c, lr, alpha, om, eps);
}

// g_stride = d_pad: every agent applies its own gradient; 0: all agents apply the same one.
__global__ __launch_bounds__(256) void rmsprop_kernel(float *x, float *v, const float *__restrict__ g, long d_pad,
                                                      long g_stride, const float *__restrict__ stats, float lr,
                                                      float alpha, float eps)
{
    const int agent = blockIdx.y;
    const float c = stats[agent * 5 + 4];
    const long n4 = d_pad / 4;
    float4 *x4 = reinterpret_cast<float4 *>(x + agent * d_pad);
    float *va = v + agent * d_pad;
    const float *ga = g + agent * g_stride;
    const float om = 1.f - alpha;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n4; i += (long)gridDim.x * 256) {
        float4 vv = stream_load4(va, i), xx = x4[i];
        // a gradient shared by all agents is read once per agent: kept cacheable
        rmsprop4(xx, vv, g_stride ? stream_load4(ga, i) : reinterpret_cast<const float4 *>(ga)[i], c, lr, alpha, om, eps);
        stream_store4(va, i, vv); x4[i] = xx;
    }
}

hipError_t launch_rmsprop(int N, const Layout &L, const HParams &hp, float *x, float *v, const float *g,
                          bool shared_gradient, const float *stats, hipStream_t s)
{
    hipLaunchKernelGGL(rmsprop_kernel, dim3(128, N), dim3(256), 0, s, x, v, g, L.d_pad,
                       shared_gradient ? 0L : L.d_pad, stats, hp.lr, hp.rms_alpha, hp.rms_eps);
    return hipGetLastError();
}

// ---- synchronous A2C with gradient averaging (Sec. 5, "Experimental setup"; Eq. (5)) --------------------
// gbar = (1/N) sum_i g_i, one thread per float4 column, agents added in index order; every
// workgroup also leaves the sum of squares of its part of gbar.
__global__ __launch_bounds__(256) void grad_mean_kernel(const float *__restrict__ g, int N, long d_pad,
                                                        float *__restrict__ gbar, float *__restrict__ part)
{
    __shared__ float red[4];
    const long n4 = d_pad / 4;
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    float ss = 0.f;
    if (e < n4) {
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
        for (int i = 0; i < N; ++i) {
            const float4 t = stream_load4(g, (long)i * n4 + e);      // every gradient is read once
            a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
        }
        const float inv = 1.f / (float)N;
        a.x *= inv; a.y *= inv; a.z *= inv; a.w *= inv;
        reinterpret_cast<float4 *>(gbar)[e] = a;
        ss = (a.x * a.x + a.y * a.y) + (a.z * a.z + a.w * a.w);
    }
    ss = block_sum_256(ss, red);
    if (threadIdx.x == 0) part[blockIdx.x] = ss;
}

// norm of gbar and the one clip factor, written into every agent's statistics row
__global__ __launch_bounds__(1024) void mean_norm_kernel(const float *__restrict__ part, int n_part, int N,
                                                         float max_norm, float *stats)
{
    __shared__ float red[16];
    float acc = 0.f;
    for (int i = threadIdx.x; i < n_part; i += 1024) acc += part[i];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    float ss = 0.f;
    for (int w = 0; w < 16; ++w) ss += red[w];
    const float norm = sqrtf(ss);
    const float c = fminf(1.f, max_norm / (norm + 1e-6f));
    for (int i = threadIdx.x; i < N; i += 1024) { stats[i * 5 + 3] = norm; stats[i * 5 + 4] = c; }
}

int grad_mean_blocks(const Layout &L) { return (int)((L.d_pad / 4 + 255) / 256); }

hipError_t launch_grad_mean(int N, const Layout &L, const HParams &hp, const float *g, float *gbar, float *part,
                            float *stats, hipStream_t s)
{
    const int blocks = grad_mean_blocks(L);
    hipLaunchKernelGGL(grad_mean_kernel, dim3(blocks), dim3(256), 0, s, g, N, L.d_pad, gbar, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mean_norm_kernel, dim3(1), dim3(1024), 0, s, part, blocks, N, hp.max_grad_norm, stats);
    return hipGetLastError();
}

// ---- gossip ------------------------------------------------------------------------------------------------
// Broadcast (Algorithm 1): keep the post-update parameters of this round for later readers.
__global__ __launch_bounds__(256) void copy_kernel(const float4 *__restrict__ src, float4 *dst, long n4)
{
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n4; i += (long)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_publish(int N, const Layout &L, const float *x, float *hist_slot, hipStream_t s)
{
    const long n4 = (long)N * L.d_pad / 4;
    const int blocks = (int)((n4 + 256 * 8 - 1) / (256 * 8));
    hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<const float4 *>(x),
                       reinterpret_cast<float4 *>(hist_slot), n4);
    return hipGetLastError();
}

// Mixing step x_i <- p_ii x_i + sum_j p_ij x_j^(round - delay_ij)  (Sec. 2; Eq. (6)).  Reads
// the pre-mix arena (and the broadcast history for delayed messages), writes the other arena,
// so every agent mixes the same snapshot.  If a delayed message was never sent the agent
// keeps its own parameters (Algorithm 1: average only when every in-peer's message is there).
constexpr int MIX_MAX_IN = 8;

// The mixing arithmetic, written with explicit roundings so that every kernel that mixes (the
// separate pass and the two fused optimizer passes) rounds in the same places whatever the
// compiler would otherwise contract: a <- w_self a, then a <- fma(w_j, m_j, a) peer by peer.
static __device__ __forceinline__ void mix_scale(float4 &a, float w)
{
    a.x = __fmul_rn(a.x, w); a.y = __fmul_rn(a.y, w); a.z = __fmul_rn(a.z, w); a.w = __fmul_rn(a.w, w);
}
static __device__ __forceinline__ void mix_add(float4 &a, float w, float4 m)
{
    a.x = __fmaf_rn(w, m.x, a.x); a.y = __fmaf_rn(w, m.y, a.y); a.z = __fmaf_rn(w, m.z, a.z); a.w = __fmaf_rn(w, m.w, a.w);
}

__global__ __launch_bounds__(256) void mix_kernel(const float *__restrict__ x_in, float *x_out,
                                                  const float *__restrict__ hist, int N, long d_pad, int tau,
                                                  long round, int phase, int max_in,
                                                  const int32_t *__restrict__ peer, const int32_t *__restrict__ delay,
                                                  const float *__restrict__ weight)
{
    const int i = blockIdx.y;
    const long tab = ((long)phase * N + i) * max_in;
    const float *src[MIX_MAX_IN];
    float w[MIX_MAX_IN];
    int n_in = 0;
    bool complete = true;
    for (int s = 0; s < max_in; ++s) {
        const int j = peer[tab + s];
        if (j < 0) continue;
        const int dl = delay[tab + s];
        const long sent = round - dl;
        if (sent < 0) { complete = false; continue; }
        src[n_in] = (dl == 0 ? x_in : hist + (sent % (tau + 1)) * (long)N * d_pad) + (long)j * d_pad;
        w[n_in] = weight[((long)phase * N + i) * (max_in + 1) + 1 + s];
        ++n_in;
    }
    const float w_self = complete ? weight[((long)phase * N + i) * (max_in + 1)] : 1.f;
    if (!complete) n_in = 0;
    const float4 *xi = reinterpret_cast<const float4 *>(x_in + (long)i * d_pad);
    float4 *xo = reinterpret_cast<float4 *>(x_out + (long)i * d_pad);
    const long n4 = d_pad / 4;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n4; e += (long)gridDim.x * 256) {
        float4 a = xi[e];
        mix_scale(a, w_self);
        for (int s = 0; s < n_in; ++s) mix_add(a, w[s], reinterpret_cast<const float4 *>(src[s])[e]);
        xo[e] = a;
    }
}

hipError_t launch_mix(int N, const Layout &L, const float *x_in, float *x_out, const float *hist, int tau,
                      long round, int phase, int max_in, const int32_t *peer, const int32_t *delay,
                      const float *weight, hipStream_t s)
{
    hipLaunchKernelGGL(mix_kernel, dim3(128, N), dim3(256), 0, s, x_in, x_out, hist, N, L.d_pad, tau, round,
                       phase, max_in, peer, delay, weight);
    return hipGetLastError();
}

// Clip + RMSprop of every agent and the mixing step in one pass (Algorithm 1: optimise,
// broadcast, average).  A workgroup owns COLS4 float4 columns of all N agents: the
// post-update parameters are kept in LDS, so a message that was sent this round is read from
// there and the parameters move through HBM once (read g, x, v; write v, x).  With delays the
// post-update values are also stored into this round's history slot and older messages are
// read from theirs.  Same arithmetic, in the same order, as rmsprop_kernel + mix_kernel.
// LDS use is N * COLS4 * 16 bytes.
constexpr int FUSED_LDS_BYTES = 64 * 1024;

template <int COLS4>
__global__ __launch_bounds__(256) void rmsprop_mix_kernel(float *x, float *v, const float *__restrict__ g,
                                                          float *hist, int N, long d_pad, int tau, long round,
                                                          int phase, int max_in, const int32_t *__restrict__ peer,
                                                          const int32_t *__restrict__ delay,
                                                          const float *__restrict__ weight,
                                                          const float *__restrict__ stats, float lr, float alpha,
                                                          float eps)
{
    extern __shared__ float4 u[];                                  // [N][COLS4]
    constexpr int GROUPS = 256 / COLS4;                            // agents in flight per pass
    const int col = threadIdx.x % COLS4;
    int q = threadIdx.x / COLS4;                                   // agents q, q + GROUPS, ...
    if constexpr (COLS4 == 64) q = __builtin_amdgcn_readfirstlane(q);   // one agent per wavefront: scalar table reads
    const long e = (long)blockIdx.x * COLS4 + col;                 // float4 index inside an agent's slice
    const long n4 = d_pad / 4;
    const float om = 1.f - alpha;
    float4 *slot = tau > 0 ? reinterpret_cast<float4 *>(hist + (round % (tau + 1)) * (long)N * d_pad) : nullptr;
    for (int i = q; i < N; i += GROUPS) {
        const long at = (long)i * n4 + e;
        float4 vv = stream_load4(v, at), xx = reinterpret_cast<float4 *>(x)[at];
        rmsprop4(xx, vv, stream_load4(g, at), stats[i * 5 + 4], lr, alpha, om, eps);
        stream_store4(v, at, vv);
        u[i * COLS4 + col] = xx;
        if (slot) slot[at] = xx;
    }
    __syncthreads();
    for (int i = q; i < N; i += GROUPS) {
        const long tab = ((long)phase * N + i) * max_in;
        bool complete = true;
        for (int s = 0; s < max_in; ++s)
            if (peer[tab + s] >= 0 && round - delay[tab + s] < 0) complete = false;
        float4 a = u[i * COLS4 + col];
        const float w_self = complete ? weight[((long)phase * N + i) * (max_in + 1)] : 1.f;
        mix_scale(a, w_self);
        if (complete)
            for (int s = 0; s < max_in; ++s) {
                const int j = peer[tab + s];
                if (j < 0) continue;
                const int dl = delay[tab + s];
                const float w = weight[((long)phase * N + i) * (max_in + 1) + 1 + s];
                const float4 m = dl == 0 ? u[j * COLS4 + col]
                                         : reinterpret_cast<const float4 *>(
                                               hist + ((round - dl) % (tau + 1)) * (long)N * d_pad)[(long)j * n4 + e];
                mix_add(a, w, m);
            }
        reinterpret_cast<float4 *>(x)[(long)i * n4 + e] = a;
    }
}

// The same pass without LDS for topologies in which every agent has exactly one in-peer, no
// delay, and the peers form a permutation (directed ring, 1-peer exponential graph): the
// permutation splits the agents into cycles a_0 <- a_1 <- ... <- a_0 (a_t receives from a_{t+1}).
// A thread owns one float4 column of one cycle and walks it once, keeping the previous agent's
// post-update value in registers, so that every value is read and written exactly once and no
// workgroup ever waits: x_new(a_t) = w_self u(a_t) + w_peer u(a_{t+1}), same order of operations
// as rmsprop_kernel + mix_kernel.  order[] lists the agents cycle by cycle, cstart[] the cycles'
// first entries (n_cycles + 1 values), both for the phase of this round.
__global__ __launch_bounds__(256) void rmsprop_mix_cycle_kernel(float *x, float *v, const float *__restrict__ g,
                                                                long d_pad, long e_begin, long e_end,
                                                                const int32_t *__restrict__ order,
                                                                const int32_t *__restrict__ cstart,
                                                                const float *__restrict__ weight,
                                                                const float *__restrict__ stats, float lr, float alpha,
                                                                float eps)
{
    const long n4 = d_pad / 4;
    const long e = e_begin + (long)blockIdx.x * 256 + threadIdx.x;       // float4 column inside an agent's slice
    if (e >= e_end) return;
    const int b0 = cstart[blockIdx.y], b1 = cstart[blockIdx.y + 1];
    const float om = 1.f - alpha;
    auto update = [&](int agent) -> float4 {
        const long at = (long)agent * n4 + e;
        float4 vv = stream_load4(v, at), xx = reinterpret_cast<float4 *>(x)[at];
        rmsprop4(xx, vv, stream_load4(g, at), stats[agent * 5 + 4], lr, alpha, om, eps);
        stream_store4(v, at, vv);
        return xx;
    };
    auto mix_store = [&](int agent, float4 own, float4 msg) {
        const float ws = weight[agent * 2], wp = weight[agent * 2 + 1];
        float4 a = own;
        mix_scale(a, ws);
        mix_add(a, wp, msg);
        reinterpret_cast<float4 *>(x)[(long)agent * n4 + e] = a;
    };
    int prev_agent = order[b0];
    const float4 first = update(prev_agent);
    float4 prev = first;
    for (int t = b0 + 1; t < b1; ++t) {
        const int agent = order[t];
        const float4 cur = update(agent);
        mix_store(prev_agent, prev, cur);
        prev = cur; prev_agent = agent;
    }
    mix_store(prev_agent, prev, first);
}

// Parameters [col_begin, col_end) (floats, multiples of 4) of every agent's slice; the whole slice by default.
hipError_t launch_rmsprop_mix_cycles(int N, const Layout &L, const HParams &hp, float *x, float *v, const float *g,
                                     const int32_t *order, const int32_t *cstart, int n_cycles, const float *weight,
                                     const float *stats, hipStream_t s, long col_begin, long col_end)
{
    if (col_end < 0) col_end = L.d_pad;
    const long e0 = col_begin / 4, e1 = col_end / 4;
    if (e1 <= e0) return hipSuccess;
    const int blocks = (int)((e1 - e0 + 255) / 256);
    hipLaunchKernelGGL(rmsprop_mix_cycle_kernel, dim3(blocks, n_cycles), dim3(256), 0, s, x, v, g, L.d_pad, e0, e1, order,
                       cstart, weight, stats, hp.lr, hp.rms_alpha, hp.rms_eps);
    (void)N;
    return hipGetLastError();
}

// widest column block whose LDS tile stays within FUSED_LDS_BYTES; 0 = too many agents
static int fused_cols4(int N)
{
    for (int c = 64; c >= 16; c >>= 1)
        if ((long)N * c * 16 <= FUSED_LDS_BYTES) return c;
    return 0;
}

bool fused_mix_available(int N) { return fused_cols4(N) != 0; }

hipError_t launch_rmsprop_mix(int N, const Layout &L, const HParams &hp, float *x, float *v, const float *g,
                              float *hist, int tau, long round, int phase, int max_in, const int32_t *peer,
                              const int32_t *delay, const float *weight, const float *stats, hipStream_t s)
{
    const int c4 = fused_cols4(N);
    const int blocks = (int)(L.d_pad / 4 / c4);                    // d_pad is a multiple of 256 floats
    const size_t lds = (size_t)N * c4 * sizeof(float4);
#define FUSED_LAUNCH(C4)                                                                                          \
    hipLaunchKernelGGL(rmsprop_mix_kernel<C4>, dim3(blocks), dim3(256), lds, s, x, v, g, hist, N, L.d_pad, tau,   \
                       round, phase, max_in, peer, delay, weight, stats, hp.lr, hp.rms_alpha, hp.rms_eps)
    if (c4 == 64) FUSED_LAUNCH(64);
    else if (c4 == 32) FUSED_LAUNCH(32);
    else if (c4 == 16) FUSED_LAUNCH(16);
    else return hipErrorInvalidValue;
#undef FUSED_LAUNCH
    return hipGetLastError();
}

// ---- distance from consensus (Prop. 1) --------------------------------------------------------------------
// A thread owns float4 columns e, e + stride, ...: for each it forms the mean over the agents (in
// double, so that identical rows give it back exactly) and adds every agent's squared deviation to
// that agent's accumulator, which it keeps in registers across its columns.  Up to CONS_KEEP agents'
// values of a column stay in registers between the two steps, so the parameters cross HBM once;
// rows beyond that are read a second time (from cache).  At the end each wavefront reduces its
// accumulators and stores one partial per agent: part[agent][block * 4 + wave].  No LDS, no
// barrier; the order of every sum is fixed by the launch shape.
constexpr int CONS_KEEP = 32;

template <int NACC>      // agents' accumulators a thread holds: 32 or 64 (NACC >= N)
__global__ __launch_bounds__(256) void consensus_kernel(const float *__restrict__ x, int N, long d_pad, int parts,
                                                        float *part)
{
    const long n4 = d_pad / 4;
    constexpr int CHUNK = 8;                             // rows beyond CONS_KEEP are taken this many at a time
    // row i of column e: uniform row pointer (scalar registers) + the thread's 32-bit byte offset
    auto ld = [&](int i, unsigned boff) -> float4 {
        return *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(x + (long)min(i, N - 1) * d_pad) + boff);
    };
    float ss[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) ss[i] = 0.f;
    // Rows i >= N do not exist: their loads are redirected to the last row, so that the loop below is
    // free of branches (all loads of a batch in flight together).  The mean takes the sum of all NACC
    // loaded rows and removes the NACC - N extra copies of the last row again; sums of at most 64 single
    // precision values in double precision are exact here for identical rows, which keeps the distance
    // of agents at consensus at exactly zero.  Accumulators of rows that do not exist are never stored.
    const double extra = (double)(NACC - N), inv_n = 1.0 / (double)N;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n4; e += (long)gridDim.x * 256) {
        const unsigned boff = (unsigned)e * 16u;         // d_pad * 4 bytes stay far below 2^32
        float4 keep[CONS_KEEP];
#pragma unroll
        for (int i = 0; i < CONS_KEEP; ++i) keep[i] = ld(i, boff);
        const float4 last = ld(N - 1, boff);
        double m0 = 0.0, m1 = 0.0, m2 = 0.0, m3 = 0.0;
#pragma unroll
        for (int i = 0; i < CONS_KEEP; ++i) { m0 += keep[i].x; m1 += keep[i].y; m2 += keep[i].z; m3 += keep[i].w; }
#pragma unroll
        for (int base = CONS_KEEP; base < NACC; base += CHUNK) {
            float4 t[CHUNK];
#pragma unroll
            for (int i = 0; i < CHUNK; ++i) t[i] = ld(base + i, boff);
#pragma unroll
            for (int i = 0; i < CHUNK; ++i) { m0 += t[i].x; m1 += t[i].y; m2 += t[i].z; m3 += t[i].w; }
        }
        m0 = (m0 - extra * last.x) * inv_n; m1 = (m1 - extra * last.y) * inv_n;
        m2 = (m2 - extra * last.z) * inv_n; m3 = (m3 - extra * last.w) * inv_n;
        auto dev2 = [&](float4 v) {
            // an opaque copy: otherwise the compiler keeps the double-precision conversions of the mean's
            // pass alive for this one, which doubles the registers a column takes
            asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
            const float a = (float)(v.x - m0), b = (float)(v.y - m1), c = (float)(v.z - m2), d = (float)(v.w - m3);
            return (a * a + b * b) + (c * c + d * d);
        };
#pragma unroll
        for (int i = 0; i < CONS_KEEP; ++i) ss[i] += dev2(keep[i]);
#pragma unroll
        for (int base = CONS_KEEP; base < NACC; base += CHUNK) {
            float4 t[CHUNK];
#pragma unroll
            for (int i = 0; i < CHUNK; ++i) t[i] = ld(base + i, boff);     // second read: from cache
#pragma unroll
            for (int i = 0; i < CHUNK; ++i) ss[base + i] += dev2(t[i]);
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < NACC; ++i) {
        const float t = wave_sum(ss[i]);
        if (lane == 0 && i < N) part[(long)i * parts + blockIdx.x * 4 + wave] = t;
    }
}

// More than 64 agents: a workgroup owns 1024 element columns, forms the mean in registers and
// block-reduces every agent's squared deviation over those columns into part[agent][chunk]; the
// second pass over the agents hits cache.
__global__ __launch_bounds__(256) void consensus_wide_kernel(const float *__restrict__ x, int N, long d_pad, int chunks,
                                                             float *part)
{
    __shared__ float red[4];
    const int chunk = blockIdx.x;
    const long e = ((long)chunk * 256 + threadIdx.x) * 4;
    const bool in = e < d_pad;
    double m0 = 0.0, m1 = 0.0, m2 = 0.0, m3 = 0.0;
    if (in)
        for (int i = 0; i < N; ++i) {
            const float4 v = *reinterpret_cast<const float4 *>(x + (long)i * d_pad + e);
            m0 += v.x; m1 += v.y; m2 += v.z; m3 += v.w;
        }
    m0 /= (double)N; m1 /= (double)N; m2 /= (double)N; m3 /= (double)N;
    for (int i = 0; i < N; ++i) {
        float ss = 0.f;
        if (in) {
            const float4 v = *reinterpret_cast<const float4 *>(x + (long)i * d_pad + e);
            const float a = (float)(v.x - m0), b = (float)(v.y - m1), c = (float)(v.z - m2), d = (float)(v.w - m3);
            ss = (a * a + b * b) + (c * c + d * d);
        }
        ss = block_sum_256(ss, red);
        if (threadIdx.x == 0) part[(long)i * chunks + chunk] = ss;
    }
}

// Row sums of a [rows][cols] array of partial sums of squares and the norms made of them, in one
// workgroup of sixteen wavefronts: wavefront w sums rows w, w + 16, ... (lane l takes columns l, l + 64,
// ... in four interleaved chains, combined in a fixed order), then row_norm[i] = sqrt(row sum)
// (optional), result[0] = sqrt(largest row sum), result[1] = sqrt(total).  row_ss receives the row sums.
__global__ __launch_bounds__(1024) void row_norms_kernel(const float *__restrict__ part, int rows, int cols,
                                                         float *row_ss, float *row_norm, float *result)
{
    __shared__ float red_max[16], red_sum[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float mx = 0.f, tot = 0.f;                             // this wavefront's rows (the same in every lane)
    for (int r = wave; r < rows; r += 16) {
        const float *p = part + (long)r * cols;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        int c = lane;
        for (; c + 192 < cols; c += 256) { a0 += p[c]; a1 += p[c + 64]; a2 += p[c + 128]; a3 += p[c + 192]; }
        for (; c < cols; c += 64) a0 += p[c];
        const float ss = wave_sum((a0 + a1) + (a2 + a3));
        if (lane == 0) {
            row_ss[r] = ss;
            if (row_norm) row_norm[r] = sqrtf(ss);
        }
        mx = fmaxf(mx, ss);
        tot += ss;
    }
    if (lane == 0) { red_max[wave] = mx; red_sum[wave] = tot; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = 0.f, t = 0.f;
        for (int w = 0; w < 16; ++w) { m = fmaxf(m, red_max[w]); t += red_sum[w]; }
        result[0] = sqrtf(m);
        result[1] = sqrtf(t);
    }
}

hipError_t launch_row_norms(const float *part, int rows, int cols, float *row_ss, float *row_norm, float *result,
                            hipStream_t s)
{
    hipLaunchKernelGGL(row_norms_kernel, dim3(1), dim3(1024), 0, s, part, rows, cols, row_ss, row_norm, result);
    return hipGetLastError();
}

// Launch shape of the register-resident kernel: every thread takes the same number of columns (the
// fewest that keeps the grid within CONS_BLOCKS workgroups), so that no wavefront runs a longer loop
// than the others.
static int consensus_blocks(const Layout &L)
{
    const long want = (L.d_pad / 4 + 255) / 256;         // workgroups at one column per thread
    const long per = (want + CONS_BLOCKS - 1) / CONS_BLOCKS;
    return (int)((want + per - 1) / per);
}

int consensus_parts(int N, const Layout &L)
{
    return N <= CONS_REG_AGENTS ? consensus_blocks(L) * 4 : (int)((L.d_pad + 1023) / 1024);
}

hipError_t launch_consensus(int N, const Layout &L, const float *x, float *part, float *row_ss, float *result,
                            hipStream_t s)
{
    const int parts = consensus_parts(N, L);
    if (N <= 32)
        hipLaunchKernelGGL(consensus_kernel<32>, dim3(parts / 4), dim3(256), 0, s, x, N, L.d_pad, parts, part);
    else if (N <= CONS_REG_AGENTS)
        hipLaunchKernelGGL(consensus_kernel<CONS_REG_AGENTS>, dim3(parts / 4), dim3(256), 0, s, x, N, L.d_pad, parts, part);
    else
        hipLaunchKernelGGL(consensus_wide_kernel, dim3(parts), dim3(256), 0, s, x, N, L.d_pad, parts, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_row_norms(part, N, parts, row_ss, nullptr, result, s);
}

// ---- canonical <-> internal order --------------------------------------------------------------------------
SegmentTable make_segments(const Layout &L)
{
    SegmentTable t{};
    long canon = 0;
    int n = 0;
    auto add = [&](long intern, int d0, int d1, int d2, int d3, long s0, long s1, long s2, long s3) {
        Segment &g = t.s[n++];
        g.canon_off = canon; g.intern_off = intern;
        g.dim[0] = d0; g.dim[1] = d1; g.dim[2] = d2; g.dim[3] = d3;
        g.stride[0] = s0; g.stride[1] = s1; g.stride[2] = s2; g.stride[3] = s3;
        g.count = (long)d0 * d1 * d2 * d3;
        canon += g.count;
    };
    // canonical OIHW -> w1 [(c, kh, kw)][o]
    add(L.w1, C1, C0, K1, K1, 1, (long)K1 * K1 * C1, (long)K1 * C1, C1);
    add(L.b1, 1, 1, 1, C1, 0, 0, 0, 1);
    // canonical OIHW -> w2 [(kh, kw, c)][o]
    add(L.w2, C2, C1, K2, K2, 1, C2, (long)K2 * C1 * C2, (long)C1 * C2);
    add(L.b2, 1, 1, 1, C2, 0, 0, 0, 1);
    add(L.w3, C3, C2, K3, K3, 1, C3, (long)K3 * C2 * C3, (long)C2 * C3);
    add(L.b3, 1, 1, 1, C3, 0, 0, 0, 1);
    // canonical [j][c][hw] -> fcw [j][hw][c]
    add(L.fcw, FC, C3, P3, 1, FLAT, 1, C3, 0);
    add(L.fcb, 1, 1, 1, FC, 0, 0, 0, 1);
    add(L.piw, 1, 1, L.n_actions, FC, 0, 0, FC, 1);
    add(L.pib, 1, 1, 1, L.n_actions, 0, 0, 0, 1);
    add(L.vw, 1, 1, 1, FC, 0, 0, 0, 1);
    add(L.vb, 1, 1, 1, 1, 0, 0, 0, 1);
    return t;
}

__global__ __launch_bounds__(256) void permute_kernel(SegmentTable tab, long d, long d_pad, float *canon,
                                                      float *intern, int to_internal)
{
    const int agent = blockIdx.y;
    const long c = (long)blockIdx.x * 256 + threadIdx.x;
    if (c >= d) return;
    int si = 0;
#pragma unroll
    for (int k = 1; k < N_SEGMENTS; ++k) if (c >= tab.s[k].canon_off) si = k;
    const Segment &g = tab.s[si];
    long r = c - g.canon_off;
    const int i3 = (int)(r % g.dim[3]); r /= g.dim[3];
    const int i2 = (int)(r % g.dim[2]); r /= g.dim[2];
    const int i1 = (int)(r % g.dim[1]); r /= g.dim[1];
    const int i0 = (int)r;
    const long ii = g.intern_off + i0 * g.stride[0] + i1 * g.stride[1] + i2 * g.stride[2] + i3 * g.stride[3];
    if (to_internal) intern[agent * d_pad + ii] = canon[agent * d + c];
    else canon[agent * d + c] = intern[agent * d_pad + ii];
}

hipError_t launch_permute(int N, const Layout &L, const SegmentTable &tab, float *canon, float *intern,
                          int to_internal, hipStream_t s)
{
    const int blocks = (int)((L.d + 255) / 256);
    hipLaunchKernelGGL(permute_kernel, dim3(blocks, N), dim3(256), 0, s, tab, L.d, L.d_pad, canon, intern,
                       to_internal);
    return hipGetLastError();
}

}  // namespace gala
