// Host side of libgala: context, arena allocation, topology tables, and the C ABI
// declared in include/gala.h.  Every numerical step is enqueued as a HIP kernel; this
// file only validates arguments, owns memory and orders launches.
#include "gala.h"
#include "gala_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

using namespace gala;

struct gala_ctx {
    int N = 0;
    Layout L{};
    SegmentTable seg{};
    HParams hp{};
    int M = 0, F = 0;
    int topo_kind = 0, tau = 0, n_phases = 1, max_in = 1;
    std::vector<int32_t> h_peer, h_delay;
    std::vector<float> h_weight;
    // one in-peer per agent, no delay, peers a permutation in every phase: its cycles, agent by agent
    bool cycles_ok = false;
    std::vector<int32_t> h_cyc_order, h_cyc_start, n_cycles;
    Buffers b{};
    int cur = 0;                 // which of b.x[] holds the current parameters
    float *canon = nullptr;      // [N][d] staging for get/set through host pointers
    int64_t last_round = -1;
    bool params_set = false;        // gala_set_params has been called: a learner step has something to learn from
    bool check_actions = false;     // GALA_CHECK_ACTIONS was set at creation: validate the action buffer of every step
    int32_t *bad_actions = nullptr; // device counter of the validation kernel
    float *scratch = nullptr;       // this device's address of the library's static scratch array
    bool shared_gradient = false;   // the last optimiser step applied the averaged gradient
    // GALA_OVERLAP_OPTIMIZER at creation: gala_round puts the hidden layer's share of its optimizer + mixing
    // pass on the side stream, where it runs beside the convolutions of the next round's forward pass
    bool overlap_optimizer = false;
    bool opt_pending = false;       // that share has been enqueued and the context's stream has not waited for it yet
    hipStream_t stream = nullptr;
    int device = 0;
    std::vector<void *> allocs;
    PhaseTimer timer;
    SideStream side;             // weight gradients run here next to the data-gradient chain
    char err[512] = {0};
};

static char g_create_err[512] = "";

static int fail(gala_ctx *c, int code, const char *fmt, ...)
{
    char *dst = c ? c->err : g_create_err;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 512, fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_OK(c, expr)                                                                          \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return fail((c), e_ == hipErrorOutOfMemory ? GALA_ENOMEM : GALA_EHIP, "%s: %s", #expr, \
                        hipGetErrorString(e_));                                                  \
    } while (0)

// Scratch memory for the entry point that must not allocate (gala_consensus_distance_noalloc): a
// file-scope device array, one copy per GPU the library runs on, held until the process ends.  In host
// code its name is only a handle: the device address is asked for once per device, with that device
// current (gala_create does it), and only that address is ever passed to kernels.
constexpr size_t SCRATCH_FLOATS = 256 * 1024;                           // 1 MiB
static __device__ __align__(256) float scratch[SCRATCH_FLOATS];
constexpr int MAX_DEVICES = 64;
static float *g_scratch_ptr[MAX_DEVICES] = {nullptr};

// Address of the scratch array on the current device (`device` is its ordinal), looked up on first use.
static hipError_t scratch_address(int device, float **out)
{
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[device]) {
        float *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

static uint64_t splitmix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Bytes from the start of the largest activation buffer (zero page included) to its end.
static unsigned long long max_buffer_bytes(int n_agents, int T, int B)
{
    const unsigned long long frames = (unsigned long long)n_agents * ((unsigned long long)T * B + B);
    return frames * A1SZ * 4ull + ZERO_PAGE * 4ull;
}

template <class T>
static int dev_alloc(gala_ctx *c, T **p, size_t count, bool zero)
{
    void *q = nullptr;
    const size_t bytes = (count ? count : 1) * sizeof(T);
    HIP_OK(c, hipMalloc(&q, bytes));
    c->allocs.push_back(q);
    if (zero) HIP_OK(c, hipMemsetAsync(q, 0, bytes, c->stream));
    *p = static_cast<T *>(q);
    return GALA_OK;
}

static int build_topology(gala_ctx *c, const gala_topology *t)
{
    const int N = c->N;
    c->topo_kind = t->kind;
    c->tau = t->max_delay;
    if (t->max_delay < 0 || t->max_delay > 16) return fail(nullptr, GALA_EINVAL, "max_delay must be in [0, 16]");
    if (t->kind == GALA_TOPO_RING) {
        c->n_phases = 1; c->max_in = 1;
    } else if (t->kind == GALA_TOPO_EXP || t->kind == GALA_TOPO_EXP_REVERSE) {
        if (N & (N - 1)) return fail(nullptr, GALA_EINVAL, "exponential graph needs a power-of-two agent count, got %d", N);
        int m = 0;
        while ((1 << (m + 1)) <= N) ++m;
        c->n_phases = m > 0 ? m : 1; c->max_in = 1;
    } else if (t->kind == GALA_TOPO_EXPLICIT) {
        if (!t->peers || !t->weights || t->n_phases < 1 || t->max_in < 1 || t->max_in > 8)
            return fail(nullptr, GALA_EINVAL, "explicit topology needs peers, weights, n_phases >= 1, 1 <= max_in <= 8");
        c->n_phases = t->n_phases; c->max_in = t->max_in;
    } else {
        return fail(nullptr, GALA_EINVAL, "unknown topology kind %d", t->kind);
    }
    const int P = c->n_phases, K = c->max_in;
    c->h_peer.assign((size_t)P * N * K, -1);
    c->h_delay.assign((size_t)P * N * K, 0);
    c->h_weight.assign((size_t)P * N * (K + 1), 0.f);
    for (int ph = 0; ph < P; ++ph)
        for (int i = 0; i < N; ++i) {
            float *w = &c->h_weight[((size_t)ph * N + i) * (K + 1)];
            int32_t *pr = &c->h_peer[((size_t)ph * N + i) * K];
            if (t->kind == GALA_TOPO_EXPLICIT) {
                double sum = 0.0;
                for (int s = 0; s <= K; ++s) {
                    w[s] = t->weights[((size_t)ph * N + i) * (K + 1) + s];
                    if (!(w[s] >= 0.f)) return fail(nullptr, GALA_EINVAL, "negative mixing weight");
                    sum += w[s];
                }
                for (int s = 0; s < K; ++s) {
                    pr[s] = t->peers[((size_t)ph * N + i) * K + s];
                    if (pr[s] >= N) return fail(nullptr, GALA_EINVAL, "peer index out of range");
                    if (pr[s] < 0) { pr[s] = -1; sum -= w[1 + s]; w[1 + s] = 0.f; }
                }
                if (std::fabs(sum - 1.0) > 1e-5)
                    return fail(nullptr, GALA_EINVAL, "mixing weights of agent %d, phase %d sum to %g, not 1", i, ph, sum);
            } else {
                // |N_in| = 1: uniform weights 1/(1+|N_in|) = 1/2 (Algorithm 1, footnote)
                pr[0] = t->kind == GALA_TOPO_RING ? (i + N - 1) % N
                      : t->kind == GALA_TOPO_EXP ? (i + (1 << ph)) % N : (i + N - (1 << ph) % N) % N;
                if (N == 1) pr[0] = 0;
                w[0] = 0.5f; w[1] = 0.5f;
            }
            for (int s = 0; s < K; ++s) {
                const uint64_t edge = ((uint64_t)ph * (uint64_t)N + (uint64_t)i) * (uint64_t)K + (uint64_t)s;
                c->h_delay[((size_t)ph * N + i) * K + s] =
                    c->tau > 0 ? (int32_t)(splitmix64(t->delay_seed + edge) % (uint64_t)(c->tau + 1)) : 0;
            }
        }
    // cycle decomposition of the peer permutation (used by the fused optimizer + mix pass)
    c->cycles_ok = K == 1 && c->tau == 0;
    c->h_cyc_order.assign((size_t)P * N, 0);
    c->h_cyc_start.assign((size_t)P * (N + 1), 0);
    c->n_cycles.assign(P, 0);
    for (int ph = 0; ph < P && c->cycles_ok; ++ph) {
        const int32_t *pr = &c->h_peer[(size_t)ph * N];
        std::vector<char> hit(N, 0), seen(N, 0);
        for (int i = 0; i < N; ++i) {
            if (pr[i] < 0 || hit[pr[i]]) { c->cycles_ok = false; break; }
            hit[pr[i]] = 1;
        }
        if (!c->cycles_ok) break;
        int pos = 0, nc = 0;
        for (int i = 0; i < N; ++i) {
            if (seen[i]) continue;
            c->h_cyc_start[(size_t)ph * (N + 1) + nc++] = pos;
            for (int a = i; !seen[a]; a = pr[a]) { seen[a] = 1; c->h_cyc_order[(size_t)ph * N + pos++] = a; }
        }
        c->h_cyc_start[(size_t)ph * (N + 1) + nc] = pos;
        c->n_cycles[ph] = nc;
    }
    return GALA_OK;
}

extern "C" int gala_create(gala_ctx **out, int n_agents, const gala_topology *topo, const gala_net_dims *net,
                           const gala_hparams *hp, void *hip_stream)
{
    if (!out || !topo || !net || !hp) return fail(nullptr, GALA_EINVAL, "null argument");
    *out = nullptr;
    if (n_agents < 1 || n_agents > 4096) return fail(nullptr, GALA_EINVAL, "n_agents must be in [1, 4096]");
    if (net->in_c != C0 || net->in_h != H0 || net->in_w != W0 || net->c1 != C1 || net->c2 != C2 ||
        net->c3 != C3 || net->fc != FC)
        return fail(nullptr, GALA_EINVAL, "only the 4x84x84 -> 32/64/64 -> 512 network is supported");
    if (net->n_actions < 1 || net->n_actions > 64) return fail(nullptr, GALA_EINVAL, "n_actions must be in [1, 64]");
    if (hp->T < 1 || hp->B < 1 || (long)hp->T * hp->B > 4096) return fail(nullptr, GALA_EINVAL, "need T, B >= 1 and T*B <= 4096");
    // the convolution kernels address an agent's activations by 32-bit byte offsets from the start of
    // the whole buffer; the largest buffer is the first layer's activations over all frames
    if (max_buffer_bytes(n_agents, hp->T, hp->B) >= (1ull << 32))
        return fail(nullptr, GALA_EINVAL, "n_agents * (T*B + B) = %lld frames exceed the 32-bit activation offsets "
                    "(at most %lld frames in one context)", (long long)n_agents * ((long long)hp->T * hp->B + hp->B),
                    (long long)(((1ull << 32) - ZERO_PAGE * 4) / ((unsigned long long)A1SZ * 4)));
    if (hp->compute_dtype != 0 && hp->compute_dtype != 1)
        return fail(nullptr, GALA_EINVAL, "compute_dtype %d not available (0 = fp32, 1 = bf16 MFMA)", hp->compute_dtype);
    if (!(hp->rms_eps > 0.f) || !(hp->rms_alpha >= 0.f && hp->rms_alpha < 1.f) || !(hp->max_grad_norm > 0.f))
        return fail(nullptr, GALA_EINVAL, "need rms_eps > 0, 0 <= rms_alpha < 1, max_grad_norm > 0");

    gala_ctx *c = new (std::nothrow) gala_ctx();
    if (!c) return fail(nullptr, GALA_ENOMEM, "out of host memory");
    c->N = n_agents;
    c->L = make_layout(net->n_actions);
    c->seg = make_segments(c->L);
    // the weight-gradient reduction writes each bias gradient right behind its weight gradient
    if (c->L.b1 != c->L.w1 + (long)KW1 * C1 || c->L.b2 != c->L.w2 + (long)KW2 * C2 ||
        c->L.b3 != c->L.w3 + (long)KW3 * C3 || c->L.fcb != c->L.fcw + (long)FC * FLAT) {
        delete c;
        return fail(nullptr, GALA_EINVAL, "internal layout: bias does not follow its weight tensor");
    }
    c->hp = HParams{hp->T, hp->B, hp->gamma, hp->vf_coef, hp->ent_coef, hp->lr, hp->rms_alpha, hp->rms_eps,
                    hp->max_grad_norm, hp->compute_dtype};
    c->M = hp->T * hp->B;
    c->F = c->M + hp->B;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->timer.stream = c->stream;
    int rc = build_topology(c, topo);
    if (rc != GALA_OK) { delete c; return rc; }

    auto bail = [&](int code) { snprintf(g_create_err, 512, "%s", c->err); gala_destroy(c); return code; };
    hipError_t he = hipGetDevice(&c->device);
    if (he != hipSuccess) { fail(c, GALA_EHIP, "hipGetDevice: %s", hipGetErrorString(he)); return bail(GALA_EHIP); }

    const size_t N = c->N, M = c->M, F = c->F, A = net->n_actions, dp = c->L.d_pad;
    Buffers &b = c->b;
#define ALLOC(ptr, count, zero) do { rc = dev_alloc(c, &(ptr), (count), (zero)); if (rc != GALA_OK) return bail(rc); } while (0)
    ALLOC(b.x[0], N * dp, true); ALLOC(b.x[1], N * dp, true);
    ALLOC(b.g, N * dp, true); ALLOC(b.v, N * dp, true);
    if (c->tau > 0) ALLOC(b.hist, (size_t)(c->tau + 1) * N * dp, true);
    // activation / gradient buffers: ZERO_PAGE zeros, then the data
#define ALLOC_ZP(ptr, count) do { ALLOC(ptr, (count) + ZERO_PAGE, false); \
        he = hipMemsetAsync((ptr), 0, ZERO_PAGE * sizeof(float), c->stream); \
        if (he != hipSuccess) { fail(c, GALA_EHIP, "zero page: %s", hipGetErrorString(he)); return bail(GALA_EHIP); } \
        (ptr) += ZERO_PAGE; } while (0)
    ALLOC_ZP(b.a1, N * F * A1SZ); ALLOC_ZP(b.a2, N * F * A2SZ);
    ALLOC_ZP(b.a3, N * F * A3SZ); ALLOC_ZP(b.h, N * F * FC);
    ALLOC(b.logits, N * M * A, true); ALLOC(b.values, N * F, true);
    ALLOC(b.ret, N * M, true); ALLOC(b.adv, N * M, true);
    ALLOC(b.dlogits, N * M * A, false); ALLOC(b.dvalues, N * M, false); ALLOC(b.loss_part, N * M * 3, false);
    ALLOC_ZP(b.dzh, N * M * FC); ALLOC_ZP(b.dz3, N * M * A3SZ);
    ALLOC_ZP(b.dz2, N * M * A2SZ); ALLOC_ZP(b.dz1, N * M * A1SZ);
#undef ALLOC_ZP
    ALLOC(b.ws, workspace_floats(c->N, c->M, c->F), false);
    ALLOC(b.norm_part, N * NORM_PARTS, true);
    ALLOC(b.gram_part, (size_t)gram_pairs(c->N) * gram_chunks(c->N) * GRAM_T * GRAM_T, false);
    ALLOC(b.gram, N * N, true); ALLOC(b.cosm, N * N, true);
    ALLOC(b.upd_part, N * UPDATE_NORM_BLOCKS, true); ALLOC(b.upd_norm, N + 2, true); ALLOC(b.row_ss, N, true);
    ALLOC(b.gbar, dp, true); ALLOC(b.gbar_part, (size_t)grad_mean_blocks(c->L), true);
    ALLOC(b.stats, N * 5, true);
    ALLOC(b.cons_part, N * (size_t)consensus_parts(c->N, c->L) + 2, true);
    ALLOC(b.peer, c->h_peer.size(), false); ALLOC(b.delay, c->h_delay.size(), false);
    ALLOC(b.weight, c->h_weight.size(), false);
    ALLOC(b.cyc_order, c->h_cyc_order.size(), false); ALLOC(b.cyc_start, c->h_cyc_start.size(), false);
    ALLOC(c->canon, N * c->L.d, false);
    ALLOC(c->bad_actions, 1, true);
#undef ALLOC
    c->check_actions = getenv("GALA_CHECK_ACTIONS") != nullptr;
    he = scratch_address(c->device, &c->scratch);
    if (he != hipSuccess) { fail(c, GALA_EHIP, "scratch array address: %s", hipGetErrorString(he)); return bail(GALA_EHIP); }
    he = hipMemcpyAsync(b.peer, c->h_peer.data(), c->h_peer.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (he == hipSuccess) he = hipMemcpyAsync(b.delay, c->h_delay.data(), c->h_delay.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (he == hipSuccess) he = hipMemcpyAsync(b.weight, c->h_weight.data(), c->h_weight.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (he == hipSuccess) he = hipMemcpyAsync(b.cyc_order, c->h_cyc_order.data(), c->h_cyc_order.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (he == hipSuccess) he = hipMemcpyAsync(b.cyc_start, c->h_cyc_start.data(), c->h_cyc_start.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (he == hipSuccess) he = hipStreamSynchronize(c->stream);
    if (he != hipSuccess) { fail(c, GALA_EHIP, "table upload: %s", hipGetErrorString(he)); return bail(GALA_EHIP); }
    if (!getenv("GALA_SINGLE_STREAM")) {
        he = hipStreamCreateWithFlags(&c->side.stream, hipStreamNonBlocking);
        // the events order two streams of this device only: no system-scope fence (host or peer visibility) when
        // one is recorded; a kernel's end still releases its writes to the device (8 us per round)
        const unsigned evf = hipEventDisableTiming | hipEventDisableSystemFence;
        for (int i = 0; i < 4 && he == hipSuccess; ++i) he = hipEventCreateWithFlags(&c->side.fork[i], evf);
        if (he == hipSuccess) he = hipEventCreateWithFlags(&c->side.join, evf);
        if (he == hipSuccess) he = hipEventCreateWithFlags(&c->side.opt_fork, evf);
        if (he == hipSuccess) he = hipEventCreateWithFlags(&c->side.opt_done, evf);
        c->overlap_optimizer = getenv("GALA_OVERLAP_OPTIMIZER") != nullptr;
        if (he != hipSuccess) { fail(c, GALA_EHIP, "side stream: %s", hipGetErrorString(he)); return bail(GALA_EHIP); }
    }
    *out = c;
    return GALA_OK;
}

extern "C" int gala_destroy(gala_ctx *c)
{
    if (!c) return GALA_OK;
    if (c->side.stream) (void)hipStreamSynchronize(c->side.stream);
    if (c->stream || !c->allocs.empty()) (void)hipStreamSynchronize(c->stream);
    for (hipEvent_t e : c->side.fork) if (e) (void)hipEventDestroy(e);
    if (c->side.join) (void)hipEventDestroy(c->side.join);
    if (c->side.opt_fork) (void)hipEventDestroy(c->side.opt_fork);
    if (c->side.opt_done) (void)hipEventDestroy(c->side.opt_done);
    if (c->side.stream) (void)hipStreamDestroy(c->side.stream);
    for (void *p : c->allocs) (void)hipFree(p);
    for (hipEvent_t e : c->timer.ev) (void)hipEventDestroy(e);
    delete c;
    return GALA_OK;
}

extern "C" size_t gala_param_count(const gala_ctx *c) { return c ? (size_t)c->L.d : 0; }

extern "C" const char *gala_last_error(const gala_ctx *c) { return c ? c->err : g_create_err; }

// The hidden layer's share of the last gala_round's optimizer pass may still be running on the side
// stream: everything that reads or writes parameters or optimizer state orders itself behind it.
static int join_optimizer(gala_ctx *c)
{
    if (c->opt_pending) {
        HIP_OK(c, hipStreamWaitEvent(c->stream, c->side.opt_done, 0));
        c->opt_pending = false;
    }
    return GALA_OK;
}
#define JOIN_OPT(c) do { int rc_ = join_optimizer(c); if (rc_ != GALA_OK) return rc_; } while (0)

// canonical [N][d] <-> an internal arena
static int export_arena(gala_ctx *c, const float *arena, float *dst, int dst_is_device)
{
    if (!c || !dst) return fail(c, GALA_EINVAL, "null argument");
    JOIN_OPT(c);
    float *stage = dst_is_device ? dst : c->canon;
    HIP_OK(c, launch_permute(c->N, c->L, c->seg, stage, const_cast<float *>(arena), 0, c->stream));
    if (!dst_is_device) {
        HIP_OK(c, hipMemcpyAsync(dst, stage, (size_t)c->N * c->L.d * 4, hipMemcpyDeviceToHost, c->stream));
        HIP_OK(c, hipStreamSynchronize(c->stream));
    }
    return GALA_OK;
}

static int import_arena(gala_ctx *c, float *arena, const float *src, int src_is_device)
{
    if (!c || !src) return fail(c, GALA_EINVAL, "null argument");
    JOIN_OPT(c);
    const float *stage = src;
    if (!src_is_device) {
        HIP_OK(c, hipMemcpyAsync(c->canon, src, (size_t)c->N * c->L.d * 4, hipMemcpyHostToDevice, c->stream));
        stage = c->canon;
    }
    HIP_OK(c, launch_permute(c->N, c->L, c->seg, const_cast<float *>(stage), arena, 1, c->stream));
    if (!src_is_device) HIP_OK(c, hipStreamSynchronize(c->stream));
    return GALA_OK;
}

extern "C" int gala_set_params(gala_ctx *c, const float *src, int dev)
{
    if (!c) return GALA_EINVAL;
    const int rc = import_arena(c, c->b.x[c->cur], src, dev);
    if (rc == GALA_OK) c->params_set = true;
    return rc;
}
extern "C" int gala_get_params(gala_ctx *c, float *dst, int dev) { return c ? export_arena(c, c->b.x[c->cur], dst, dev) : GALA_EINVAL; }
extern "C" int gala_set_opt_state(gala_ctx *c, const float *src, int dev) { return c ? import_arena(c, c->b.v, src, dev) : GALA_EINVAL; }
extern "C" int gala_get_opt_state(gala_ctx *c, float *dst, int dev) { return c ? export_arena(c, c->b.v, dst, dev) : GALA_EINVAL; }
extern "C" int gala_get_grads(gala_ctx *c, float *dst, int dev) { return c ? export_arena(c, c->b.g, dst, dev) : GALA_EINVAL; }

extern "C" int gala_get_mean_grad(gala_ctx *c, float *dst, int dst_is_device)
{
    if (!c || !dst) return fail(c, GALA_EINVAL, "null argument");
    float *stage = dst_is_device ? dst : c->canon;
    HIP_OK(c, launch_permute(1, c->L, c->seg, stage, c->b.gbar, 0, c->stream));
    if (!dst_is_device) {
        HIP_OK(c, hipMemcpyAsync(dst, stage, (size_t)c->L.d * 4, hipMemcpyDeviceToHost, c->stream));
        HIP_OK(c, hipStreamSynchronize(c->stream));
    }
    return GALA_OK;
}

// forward, loss, backward and the per-agent gradient norm / clip factor
static int enqueue_gradients(gala_ctx *c, const uint8_t *obs_u8, const int32_t *actions, const float *rewards,
                             const uint8_t *dones, const uint8_t *bootstrap_obs, bool own_norm = true,
                             bool late_join = false)
{
    if (!obs_u8 || !actions || !rewards || !dones || !bootstrap_obs) return fail(c, GALA_EINVAL, "null input buffer");
    if ((reinterpret_cast<uintptr_t>(obs_u8) | reinterpret_cast<uintptr_t>(bootstrap_obs)) & 3)
        return fail(c, GALA_EINVAL, "observation buffers must be 4-byte aligned");
    if (!c->params_set) return fail(c, GALA_ESTATE, "learner step before gala_set_params: the parameters are all zero");
    if (c->check_actions) {
        // opt-in (GALA_CHECK_ACTIONS): count the actions outside [0, A) and refuse the step; synchronises
        int32_t bad = 0;
        HIP_OK(c, launch_count_bad_actions(actions, (long)c->N * c->M, c->L.n_actions, c->bad_actions, c->stream));
        HIP_OK(c, hipMemcpyAsync(&bad, c->bad_actions, 4, hipMemcpyDeviceToHost, c->stream));
        HIP_OK(c, hipStreamSynchronize(c->stream));
        if (bad) return fail(c, GALA_EINVAL, "%d action(s) outside [0, %d)", (int)bad, c->L.n_actions);
    }
    NetArgs a{};
    a.N = c->N; a.M = c->M; a.F = c->F; a.Bn = c->hp.B; a.L = c->L;
    a.x = c->b.x[c->cur]; a.b = c->b; a.obs = obs_u8; a.boot = bootstrap_obs;
    a.bf16 = c->hp.compute_dtype == 1;
    PhaseTimer *pt = &c->timer;
    pt->begin();
    // a pending share of the previous optimizer pass covers the hidden layer's weights only: the
    // convolutions may start, the stream waits in front of the hidden layer (late_join) or right here
    hipEvent_t before_fc = nullptr;
    if (c->opt_pending && late_join) { before_fc = c->side.opt_done; c->opt_pending = false; }
    else JOIN_OPT(c);
    HIP_OK(c, launch_forward(a, c->stream, pt, before_fc));
    HIP_OK(c, launch_loss(a, c->hp, actions, rewards, dones, c->stream));
    pt->mark("loss_heads_dgrad");
    HIP_OK(c, launch_backward(a, c->hp, c->stream, pt, &c->side));
    (void)own_norm;          // the backward pass always leaves every agent's own norm and clip factor in stats
    return GALA_OK;
}

static int check_round(gala_ctx *c, int64_t round)
{
    if (round < 0) return fail(c, GALA_EINVAL, "negative round");
    // delayed messages are read from the history of consecutive rounds
    if (c->tau > 0 && round != c->last_round + 1)
        return fail(c, GALA_ESTATE, "with max_delay > 0 rounds must be consecutive from 0: got %lld after %lld",
                    (long long)round, (long long)c->last_round);
    if (round < c->last_round)
        return fail(c, GALA_ESTATE, "gossip round went backwards: %lld after %lld", (long long)round, (long long)c->last_round);
    return GALA_OK;
}

extern "C" int gala_learner_step(gala_ctx *c, const uint8_t *obs_u8, const int32_t *actions, const float *rewards,
                                 const uint8_t *dones, const uint8_t *bootstrap_obs)
{
    if (!c) return GALA_EINVAL;
    int rc = enqueue_gradients(c, obs_u8, actions, rewards, dones, bootstrap_obs);
    if (rc != GALA_OK) return rc;
    HIP_OK(c, launch_rmsprop(c->N, c->L, c->hp, c->b.x[c->cur], c->b.v, c->b.g, false, c->b.stats, c->stream));
    c->timer.mark("clip_rmsprop");
    c->shared_gradient = false;
    return GALA_OK;
}

extern "C" int gala_a2c_allreduce_step(gala_ctx *c, const uint8_t *obs_u8, const int32_t *actions,
                                       const float *rewards, const uint8_t *dones, const uint8_t *bootstrap_obs)
{
    if (!c) return GALA_EINVAL;
    int rc = enqueue_gradients(c, obs_u8, actions, rewards, dones, bootstrap_obs, false);
    if (rc != GALA_OK) return rc;
    HIP_OK(c, launch_grad_mean(c->N, c->L, c->hp, c->b.g, c->b.gbar, c->b.gbar_part, c->b.stats, c->stream));
    c->timer.mark("grad_mean_norm");
    HIP_OK(c, launch_rmsprop(c->N, c->L, c->hp, c->b.x[c->cur], c->b.v, c->b.gbar, true, c->b.stats, c->stream));
    c->timer.mark("clip_rmsprop");
    c->shared_gradient = true;
    return GALA_OK;
}

extern "C" int gala_gossip(gala_ctx *c, int64_t round)
{
    if (!c) return GALA_EINVAL;
    int rc = check_round(c, round);
    if (rc != GALA_OK) return rc;
    JOIN_OPT(c);
    if (c->tau > 0) {
        float *slot = c->b.hist + (size_t)(round % (c->tau + 1)) * c->N * c->L.d_pad;
        HIP_OK(c, launch_publish(c->N, c->L, c->b.x[c->cur], slot, c->stream));
        c->timer.mark("gossip_publish");
    }
    const int phase = (int)(round % c->n_phases);
    HIP_OK(c, launch_mix(c->N, c->L, c->b.x[c->cur], c->b.x[c->cur ^ 1], c->b.hist, c->tau, (long)round, phase,
                         c->max_in, c->b.peer, c->b.delay, c->b.weight, c->stream));
    c->timer.mark("gossip_mix");
    c->cur ^= 1;
    c->last_round = round;
    return GALA_OK;
}

extern "C" int gala_round(gala_ctx *c, const uint8_t *obs_u8, const int32_t *actions, const float *rewards,
                          const uint8_t *dones, const uint8_t *bootstrap_obs, int64_t round)
{
    if (!c) return GALA_EINVAL;
    int rc = check_round(c, round);
    if (rc != GALA_OK) return rc;
    if (!c->cycles_ok && !fused_mix_available(c->N)) {
        rc = gala_learner_step(c, obs_u8, actions, rewards, dones, bootstrap_obs);
        return rc != GALA_OK ? rc : gala_gossip(c, round);
    }
    rc = enqueue_gradients(c, obs_u8, actions, rewards, dones, bootstrap_obs, true, true);
    if (rc != GALA_OK) return rc;
    const int phase = (int)(round % c->n_phases);
    if (c->cycles_ok) {
        auto pass = [&](hipStream_t s, long col0, long col1) {
            return launch_rmsprop_mix_cycles(c->N, c->L, c->hp, c->b.x[c->cur], c->b.v, c->b.g,
                                             c->b.cyc_order + (size_t)phase * c->N,
                                             c->b.cyc_start + (size_t)phase * (c->N + 1), c->n_cycles[phase],
                                             c->b.weight + (size_t)phase * c->N * 2, c->b.stats, s, col0, col1);
        };
        if (c->overlap_optimizer && c->side.stream && !c->timer.on) {
            // the hidden layer's weights (95 % of the parameters) are first read by the fourth kernel of a
            // forward pass: their share of this pass goes to the side stream, the rest stays here
            const long w0 = c->L.fcw, w1 = c->L.fcw + (long)FC * FLAT;
            HIP_OK(c, hipEventRecord(c->side.opt_fork, c->stream));
            HIP_OK(c, hipStreamWaitEvent(c->side.stream, c->side.opt_fork, 0));
            HIP_OK(c, pass(c->side.stream, w0, w1));
            HIP_OK(c, hipEventRecord(c->side.opt_done, c->side.stream));
            HIP_OK(c, pass(c->stream, 0, w0));
            HIP_OK(c, pass(c->stream, w1, c->L.d_pad));
            c->opt_pending = true;
        } else {
            HIP_OK(c, pass(c->stream, 0, c->L.d_pad));
        }
        c->timer.mark("clip_rmsprop_mix");
        c->shared_gradient = false;
        c->last_round = round;
        return GALA_OK;
    }
    HIP_OK(c, launch_rmsprop_mix(c->N, c->L, c->hp, c->b.x[c->cur], c->b.v, c->b.g, c->b.hist, c->tau, (long)round,
                                 phase, c->max_in, c->b.peer, c->b.delay, c->b.weight, c->b.stats, c->stream));
    c->timer.mark("clip_rmsprop_mix");
    c->shared_gradient = false;
    c->last_round = round;
    return GALA_OK;
}

extern "C" int gala_act(gala_ctx *c, const uint8_t *obs_u8, uint64_t seed, int64_t step, int32_t *actions,
                        float *values, float *logp)
{
    if (!c) return GALA_EINVAL;
    if (!obs_u8 || !actions) return fail(c, GALA_EINVAL, "null observation or action buffer");
    if (reinterpret_cast<uintptr_t>(obs_u8) & 3) return fail(c, GALA_EINVAL, "observation buffer must be 4-byte aligned");
    if (step < 0) return fail(c, GALA_EINVAL, "negative acting step");
    if (!c->params_set) return fail(c, GALA_ESTATE, "acting step before gala_set_params: the parameters are all zero");
    JOIN_OPT(c);
    // forward pass over B frames per agent: all of them take the policy head, none is a bootstrap state
    NetArgs a{};
    a.N = c->N; a.M = c->hp.B; a.F = c->hp.B; a.Bn = 0; a.L = c->L;
    a.x = c->b.x[c->cur]; a.b = c->b; a.obs = obs_u8; a.boot = obs_u8;
    a.bf16 = c->hp.compute_dtype == 1;
    PhaseTimer *pt = &c->timer;
    pt->begin();
    HIP_OK(c, launch_forward(a, c->stream, pt));
    HIP_OK(c, launch_sample(c->N, c->hp.B, c->L.n_actions, c->b.logits, c->b.values, seed, (long)step, actions,
                            values, logp, c->stream));
    pt->mark("sample");
    return GALA_OK;
}

extern "C" int gala_get_step_stats(gala_ctx *c, float *dst_host)
{
    if (!c || !dst_host) return fail(c, GALA_EINVAL, "null argument");
    HIP_OK(c, hipMemcpyAsync(dst_host, c->b.stats, (size_t)c->N * 5 * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    return GALA_OK;
}

extern "C" int gala_get_outputs(gala_ctx *c, float *logits, float *values, float *returns, float *advantages)
{
    if (!c) return GALA_EINVAL;
    const size_t N = c->N, M = c->M, F = c->F, A = c->L.n_actions;
    if (logits) HIP_OK(c, hipMemcpyAsync(logits, c->b.logits, N * M * A * 4, hipMemcpyDeviceToHost, c->stream));
    if (values) HIP_OK(c, hipMemcpyAsync(values, c->b.values, N * F * 4, hipMemcpyDeviceToHost, c->stream));
    if (returns) HIP_OK(c, hipMemcpyAsync(returns, c->b.ret, N * M * 4, hipMemcpyDeviceToHost, c->stream));
    if (advantages) HIP_OK(c, hipMemcpyAsync(advantages, c->b.adv, N * M * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    return GALA_OK;
}

extern "C" int gala_consensus_distance(gala_ctx *c, float *max_dist, float *frob)
{
    if (!c || !max_dist || !frob) return fail(c, GALA_EINVAL, "null argument");
    JOIN_OPT(c);
    float *result = c->b.cons_part + (size_t)c->N * consensus_parts(c->N, c->L);
    c->timer.mark("diag_begin");
    HIP_OK(c, launch_consensus(c->N, c->L, c->b.x[c->cur], c->b.cons_part, c->b.row_ss, result, c->stream));
    c->timer.mark("consensus_distance");
    float r[2];
    HIP_OK(c, hipMemcpyAsync(r, result, 8, hipMemcpyDeviceToHost, c->stream));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    *max_dist = r[0]; *frob = r[1];
    return GALA_OK;
}

extern "C" int gala_consensus_distance_noalloc(gala_ctx *c, float *result_dev)
{
    if (!c || !result_dev) return fail(c, GALA_EINVAL, "null argument");
    JOIN_OPT(c);
    // partial sums of squares [N][parts], then the row sums [N], all in the static scratch array
    const size_t need = (size_t)c->N * consensus_parts(c->N, c->L) + (size_t)c->N;
    if (need > SCRATCH_FLOATS)
        return fail(c, GALA_EINVAL, "gala_consensus_distance_noalloc: %d agents need %zu floats of scratch, the static "
                    "array holds %zu; use gala_consensus_distance", c->N, need, (size_t)SCRATCH_FLOATS);
    float *part = c->scratch, *row_ss = c->scratch + (size_t)c->N * consensus_parts(c->N, c->L);
    HIP_OK(c, launch_consensus(c->N, c->L, c->b.x[c->cur], part, row_ss, result_dev, c->stream));
    return GALA_OK;
}

extern "C" int gala_get_head_grads(gala_ctx *c, float *dlogits_host, float *dvalues_host)
{
    if (!c) return GALA_EINVAL;
    const size_t n = (size_t)c->N * c->M;
    if (dlogits_host)
        HIP_OK(c, hipMemcpyAsync(dlogits_host, c->b.dlogits, n * c->L.n_actions * 4, hipMemcpyDeviceToHost, c->stream));
    if (dvalues_host) HIP_OK(c, hipMemcpyAsync(dvalues_host, c->b.dvalues, n * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    return GALA_OK;
}

extern "C" int gala_grad_cosine(gala_ctx *c, float *cos_host)
{
    if (!c || !cos_host) return fail(c, GALA_EINVAL, "null argument");
    c->timer.mark("diag_begin");
    HIP_OK(c, launch_grad_cosine(c->N, c->L, c->b.g, c->b.gram_part, c->b.gram, c->b.cosm, c->stream));
    c->timer.mark("grad_cosine");
    HIP_OK(c, hipMemcpyAsync(cos_host, c->b.cosm, (size_t)c->N * c->N * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    return GALA_OK;
}

extern "C" int gala_update_norm(gala_ctx *c, float *row_norms_host, float *frob_host)
{
    if (!c || !frob_host) return fail(c, GALA_EINVAL, "null argument");
    JOIN_OPT(c);
    c->timer.mark("diag_begin");
    HIP_OK(c, launch_update_norm(c->N, c->L, c->hp, c->shared_gradient ? c->b.gbar : c->b.g, c->shared_gradient,
                                 c->b.v, c->b.stats, c->b.upd_part, c->b.row_ss, c->b.upd_norm, c->stream));
    c->timer.mark("update_norm");
    if (row_norms_host)
        HIP_OK(c, hipMemcpyAsync(row_norms_host, c->b.upd_norm, (size_t)c->N * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_OK(c, hipMemcpyAsync(frob_host, c->b.upd_norm + c->N + 1, 4, hipMemcpyDeviceToHost, c->stream));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    return GALA_OK;
}

extern "C" int gala_prop1_bound(double beta, const double *update_norms, int n, double *bound)
{
    if (!update_norms || !bound || n < 0 || !(beta >= 0.0 && beta <= 1.0))
        return fail(nullptr, GALA_EINVAL, "need update norms, 0 <= beta <= 1, n >= 0");
    // sum_{s < n} beta^(n - s) u_s by Horner's rule: B <- beta (B + u_s)
    double b = 0.0;
    for (int s = 0; s < n; ++s) b = beta * (b + update_norms[s]);
    *bound = b;
    return GALA_OK;
}

extern "C" int gala_get_peer_table(gala_ctx *c, int64_t round, int32_t *peer, int32_t *delay)
{
    if (!c || round < 0 || (!peer && !delay)) return fail(c, GALA_EINVAL, "bad argument");
    const int phase = (int)(round % c->n_phases);
    const size_t n = (size_t)c->N * c->max_in, off = (size_t)phase * n;
    if (peer) memcpy(peer, c->h_peer.data() + off, n * 4);
    if (delay) memcpy(delay, c->h_delay.data() + off, n * 4);
    return GALA_OK;
}

extern "C" int gala_set_profiling(gala_ctx *c, int enabled)
{
    if (!c) return GALA_EINVAL;
    JOIN_OPT(c);
    c->timer.on = enabled != 0;
    c->timer.n = 0;
    return GALA_OK;
}

extern "C" int gala_get_phase_times(gala_ctx *c, char *names, size_t names_cap, float *ms, int cap, int *n_out)
{
    if (!c || !names || !ms || !n_out || names_cap == 0) return fail(c, GALA_EINVAL, "null argument");
    HIP_OK(c, hipStreamSynchronize(c->stream));
    names[0] = 0;
    int n = 0;
    size_t used = 0;
    for (int i = 1; i < c->timer.n && n < cap; ++i) {
        float t = 0.f;
        HIP_OK(c, hipEventElapsedTime(&t, c->timer.ev[i - 1], c->timer.ev[i]));
        const size_t len = strlen(c->timer.names[i]);
        if (used + len + 2 > names_cap) break;
        memcpy(names + used, c->timer.names[i], len);
        used += len;
        names[used++] = ';';
        names[used] = 0;
        ms[n++] = t;
    }
    *n_out = n;
    return GALA_OK;
}

extern "C" int gala_get_activations(gala_ctx *c, int layer, float *dst_host)
{
    if (!c || !dst_host) return fail(c, GALA_EINVAL, "null argument");
    const float *src = nullptr;
    size_t per_frame = 0;
    switch (layer) {
    case 1: src = c->b.a1; per_frame = A1SZ; break;
    case 2: src = c->b.a2; per_frame = A2SZ; break;
    case 3: src = c->b.a3; per_frame = A3SZ; break;
    case 4: src = c->b.h; per_frame = FC; break;
    default: return fail(c, GALA_EINVAL, "layer must be 1..4");
    }
    HIP_OK(c, hipMemcpyAsync(dst_host, src, (size_t)c->N * c->F * per_frame * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    return GALA_OK;
}
