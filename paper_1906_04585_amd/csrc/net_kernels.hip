// Agent-grouped forward and backward passes of the 3-conv / 1-hidden / two-head network
// (App. C.2 of the paper) as implicit GEMMs on the fp32 matrix cores, plus the small
// kernels around them (heads, bias gradients, split-K reduction).
//
// Activations are channels-last: a1 [f][20][20][32], a2 [f][9][9][64], a3 [f][7][7][64],
// h [f][512]; frame f < M is rollout sample t*B + b, frames M..F-1 are the bootstrap
// states.  Backward buffers hold gradients w.r.t. the values *before* each ReLU.
#include "gala_internal.h"
#include "igemm.h"

namespace gala {

static __device__ __forceinline__ void ld4(float (&r)[4], const float *p)
{
    const float4 v = *reinterpret_cast<const float4 *>(p);
    r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
}

static __device__ __forceinline__ void ld4_u8(float (&r)[4], const uint8_t *p)
{
    const uint32_t w = *reinterpret_cast<const uint32_t *>(p);
    constexpr float sc = 1.0f / 255.0f;      // states are bytes scaled to [0, 1]
    r[0] = (float)(w & 255u) * sc;
    r[1] = (float)((w >> 8) & 255u) * sc;
    r[2] = (float)((w >> 16) & 255u) * sc;
    r[3] = (float)(w >> 24) * sc;
}

struct ProblemBase {
    int tiles_m, tiles_n, splits;
    int k0, k1;
    __device__ int k_begin() const { return k0; }
    __device__ int k_end() const { return k1; }
};

// ---- conv1 forward: bytes -> a1 ------------------------------------------------------
// m = (f, oy, ox), n = o, k = (c, kh, kw).
struct Conv1Fwd : ProblemBase {
    static constexpr int BM = 256, BN = 32, BK = 16, WM = 4, WN = 1;
    static constexpr bool A_KC = true, B_KC = false;
    const uint8_t *obs, *boot;
    const float *x;
    float *a1;
    long d_pad, w_off, b_off;
    int M, F, Bn;
    const uint8_t *o_, *bo_;
    const float *w_, *b_;
    float *out_;
    int rows_;
    __device__ void bind(int agent, int)
    {
        o_ = obs + (long)agent * M * FRAME;
        bo_ = boot + (long)agent * Bn * FRAME;
        w_ = x + agent * d_pad + w_off;
        b_ = x + agent * d_pad + b_off;
        out_ = a1 + (long)agent * F * A1SZ;
        rows_ = F * P1;
        k0 = 0; k1 = KW1;
    }
    __device__ void load_a(float (&r)[4], int m, int k) const
    {
        if (m >= rows_) return;
        const int f = m / P1, p = m % P1, oy = p / W1, ox = p % W1;
        const int c = k >> 6, kh = (k >> 3) & 7, kw = k & 7;
        const uint8_t *fr = f < M ? o_ + (long)f * FRAME : bo_ + (long)(f - M) * FRAME;
        ld4_u8(r, fr + c * (H0 * W0) + (oy * S1 + kh) * W0 + ox * S1 + kw);
    }
    __device__ void load_b(float (&r)[4], int k, int n) const { ld4(r, w_ + k * C1 + n); }
    __device__ void store(int m, int n, float v) const
    {
        if (m < rows_) out_[(long)m * C1 + n] = fmaxf(v + b_[n], 0.f);
    }
};

// ---- conv2 / conv3 forward ---------------------------------------------------------------
// m = (f, oy, ox), n = o, k = (kh, kw, c) over a channels-last input.
template <int CI, int HI, int WI, int CO, int HO, int WO, int KS, int ST>
struct ConvFwd : ProblemBase {
    static constexpr int BM = 128, BN = 64, BK = 16, WM = 2, WN = 2;
    static constexpr bool A_KC = true, B_KC = false;
    const float *in, *x;
    float *out;
    long d_pad, w_off, b_off;
    int F;
    const float *in_, *w_, *b_;
    float *out_;
    int rows_;
    __device__ void bind(int agent, int)
    {
        in_ = in + (long)agent * F * (HI * WI * CI);
        w_ = x + agent * d_pad + w_off;
        b_ = x + agent * d_pad + b_off;
        out_ = out + (long)agent * F * (HO * WO * CO);
        rows_ = F * HO * WO;
        k0 = 0; k1 = KS * KS * CI;
    }
    __device__ void load_a(float (&r)[4], int m, int k) const
    {
        if (m >= rows_) return;
        const int f = m / (HO * WO), p = m % (HO * WO), oy = p / WO, ox = p % WO;
        const int kh = k / (KS * CI), rem = k % (KS * CI);
        ld4(r, in_ + ((long)(f * HI + oy * ST + kh) * WI + ox * ST) * CI + rem);
    }
    __device__ void load_b(float (&r)[4], int k, int n) const { ld4(r, w_ + k * CO + n); }
    __device__ void store(int m, int n, float v) const
    {
        if (m < rows_) out_[(long)m * CO + n] = fmaxf(v + b_[n], 0.f);
    }
};
using Conv2Fwd = ConvFwd<C1, H1, W1, C2, H2, W2, K2, S2>;
using Conv3Fwd = ConvFwd<C2, H2, W2, C3, H3, W3, K3, S3>;

// ---- hidden layer forward (split over k; partial sums to the workspace) -------------------
// m = f, n = j, k = flattened a3.
struct FcFwd : ProblemBase {
    static constexpr int BM = 96, BN = 128, BK = 16, WM = 1, WN = 4;
    static constexpr bool A_KC = true, B_KC = true;
    const float *a3, *x;
    float *ws;
    long d_pad, w_off;
    int F, kchunk;
    const float *a_, *w_;
    float *out_;
    __device__ void bind(int agent, int split)
    {
        a_ = a3 + (long)agent * F * FLAT;
        w_ = x + agent * d_pad + w_off;
        out_ = ws + ((long)agent * splits + split) * F * FC;
        k0 = split * kchunk;
        k1 = min(FLAT, k0 + kchunk);
    }
    __device__ void load_a(float (&r)[4], int m, int k) const
    {
        if (m < F) ld4(r, a_ + (long)m * FLAT + k);
    }
    __device__ void load_b(float (&r)[4], int k, int n) const { ld4(r, w_ + (long)n * FLAT + k); }
    __device__ void store(int m, int n, float v) const
    {
        if (m < F) out_[(long)m * FC + n] = v;
    }
};

// ---- hidden layer: gradient to a3 (masked by its ReLU) ---------------------------------------
// m = f, n = flattened a3 index, k = j.
struct FcDgrad : ProblemBase {
    static constexpr int BM = 96, BN = 128, BK = 16, WM = 1, WN = 4;
    static constexpr bool A_KC = true, B_KC = false;
    const float *dzh, *x, *a3;
    float *dz3;
    long d_pad, w_off;
    int M, F;
    const float *a_, *w_, *act_;
    float *out_;
    __device__ void bind(int agent, int)
    {
        a_ = dzh + (long)agent * M * FC;
        w_ = x + agent * d_pad + w_off;
        act_ = a3 + (long)agent * F * FLAT;
        out_ = dz3 + (long)agent * M * FLAT;
        k0 = 0; k1 = FC;
    }
    __device__ void load_a(float (&r)[4], int m, int k) const
    {
        if (m < M) ld4(r, a_ + (long)m * FC + k);
    }
    __device__ void load_b(float (&r)[4], int k, int n) const
    {
        if (n < FLAT) ld4(r, w_ + (long)k * FLAT + n);
    }
    __device__ void store(int m, int n, float v) const
    {
        if (m < M && n < FLAT) {
            const long i = (long)m * FLAT + n;
            out_[i] = act_[i] > 0.f ? v : 0.f;
        }
    }
};

// ---- hidden layer: weight gradient ---------------------------------------------------------
// m = j, n = flattened a3 index, k = f.
struct FcWgrad : ProblemBase {
    static constexpr int BM = 128, BN = 128, BK = 16, WM = 2, WN = 2;
    static constexpr bool A_KC = false, B_KC = false;
    const float *dzh, *a3;
    float *g;
    long d_pad, w_off;
    int M, F;
    const float *a_, *b_;
    float *out_;
    __device__ void bind(int agent, int)
    {
        a_ = dzh + (long)agent * M * FC;
        b_ = a3 + (long)agent * F * FLAT;
        out_ = g + agent * d_pad + w_off;
        k0 = 0; k1 = M;
    }
    __device__ void load_a(float (&r)[4], int m, int k) const { ld4(r, a_ + (long)k * FC + m); }
    __device__ void load_b(float (&r)[4], int k, int n) const
    {
        if (n < FLAT) ld4(r, b_ + (long)k * FLAT + n);
    }
    __device__ void store(int m, int n, float v) const
    {
        if (n < FLAT) out_[(long)m * FLAT + n] = v;
    }
};

// ---- conv3: gradient to a2 (stride 1: full correlation with the flipped kernel) -----------------
// m = (f, iy, ix), n = c, k = (kh, kw, o).
struct Conv3Dgrad : ProblemBase {
    static constexpr int BM = 128, BN = 64, BK = 16, WM = 2, WN = 2;
    static constexpr bool A_KC = true, B_KC = true;
    const float *dz3, *x, *a2;
    float *dz2;
    long d_pad, w_off;
    int M, F;
    const float *a_, *w_, *act_;
    float *out_;
    int rows_;
    __device__ void bind(int agent, int)
    {
        a_ = dz3 + (long)agent * M * A3SZ;
        w_ = x + agent * d_pad + w_off;
        act_ = a2 + (long)agent * F * A2SZ;
        out_ = dz2 + (long)agent * M * A2SZ;
        rows_ = M * P2;
        k0 = 0; k1 = K3 * K3 * C3;
    }
    __device__ void load_a(float (&r)[4], int m, int k) const
    {
        if (m >= rows_) return;
        const int f = m / P2, p = m % P2, iy = p / W2, ix = p % W2;
        const int t = k / C3, o = k % C3, kh = t / K3, kw = t % K3;
        const int oy = iy - kh, ox = ix - kw;
        if (oy < 0 || oy >= H3 || ox < 0 || ox >= W3) return;
        ld4(r, a_ + ((long)(f * H3 + oy) * W3 + ox) * C3 + o);
    }
    __device__ void load_b(float (&r)[4], int k, int n) const
    {
        const int t = k / C3, o = k % C3;
        ld4(r, w_ + ((long)t * C2 + n) * C3 + o);
    }
    __device__ void store(int m, int n, float v) const
    {
        if (m < rows_) {
            const long i = (long)m * C2 + n;
            out_[i] = act_[i] > 0.f ? v : 0.f;
        }
    }
};

// ---- conv2: gradient to a1 (stride 2) ----------------------------------------------------------
// Input positions split into four parity classes (iy%2, ix%2), carried in the "split"
// index; within a class the transposed convolution is a stride-1 2x2 correlation:
// m = (f, y', x') with iy = 2y'+py, n = c, k = (a, b, o) with kh = py + 2a, oy = y' - a.
struct Conv2Dgrad : ProblemBase {
    static constexpr int BM = 256, BN = 32, BK = 16, WM = 4, WN = 1;
    static constexpr bool A_KC = true, B_KC = true;
    static constexpr int HY = H1 / 2, WX = W1 / 2, PC = HY * WX;   // 10, 10, 100
    const float *dz2, *x, *a1;
    float *dz1;
    long d_pad, w_off;
    int M, F;
    const float *a_, *w_, *act_;
    float *out_;
    int rows_, py_, px_;
    __device__ void bind(int agent, int cls)
    {
        a_ = dz2 + (long)agent * M * A2SZ;
        w_ = x + agent * d_pad + w_off;
        act_ = a1 + (long)agent * F * A1SZ;
        out_ = dz1 + (long)agent * M * A1SZ;
        rows_ = M * PC;
        py_ = cls >> 1; px_ = cls & 1;
        k0 = 0; k1 = 4 * C2;
    }
    __device__ void load_a(float (&r)[4], int m, int k) const
    {
        if (m >= rows_) return;
        const int f = m / PC, p = m % PC, yy = p / WX, xx = p % WX;
        const int t = k / C2, o = k % C2, a = t >> 1, b = t & 1;
        const int oy = yy - a, ox = xx - b;
        if (oy < 0 || oy >= H2 || ox < 0 || ox >= W2) return;
        ld4(r, a_ + ((long)(f * H2 + oy) * W2 + ox) * C2 + o);
    }
    __device__ void load_b(float (&r)[4], int k, int n) const
    {
        const int t = k / C2, o = k % C2, a = t >> 1, b = t & 1;
        const int kh = py_ + 2 * a, kw = px_ + 2 * b;
        ld4(r, w_ + ((long)(kh * K2 + kw) * C1 + n) * C2 + o);
    }
    __device__ void store(int m, int n, float v) const
    {
        if (m < rows_) {
            const int f = m / PC, p = m % PC, yy = p / WX, xx = p % WX;
            const long i = ((long)(f * H1 + 2 * yy + py_) * W1 + 2 * xx + px_) * C1 + n;
            out_[i] = act_[i] > 0.f ? v : 0.f;
        }
    }
};

// ---- conv2 / conv3 weight gradient (split over frames) ----------------------------------------------
// m = (kh, kw, c), n = o, k = (f, oy, ox).
template <int CI, int HI, int WI, int CO, int HO, int WO, int KS, int ST, int BM_>
struct ConvWgrad : ProblemBase {
    static constexpr int BM = BM_, BN = 64, BK = 16, WM = 2, WN = 2;
    static constexpr bool A_KC = false, B_KC = false;
    static constexpr int MT = KS * KS * CI;
    const float *in, *dz;
    float *ws;
    int M, F, fps;
    const float *in_, *dz_;
    float *out_;
    __device__ void bind(int agent, int split)
    {
        in_ = in + (long)agent * F * (HI * WI * CI);
        dz_ = dz + (long)agent * M * (HO * WO * CO);
        out_ = ws + ((long)agent * splits + split) * MT * CO;
        k0 = split * fps * (HO * WO);
        k1 = min(M, (split + 1) * fps) * (HO * WO);
    }
    __device__ void load_a(float (&r)[4], int m, int k) const
    {
        if (m >= MT) return;
        const int f = k / (HO * WO), p = k % (HO * WO), oy = p / WO, ox = p % WO;
        const int kh = m / (KS * CI), rem = m % (KS * CI);
        ld4(r, in_ + ((long)(f * HI + oy * ST + kh) * WI + ox * ST) * CI + rem);
    }
    __device__ void load_b(float (&r)[4], int k, int n) const { ld4(r, dz_ + (long)k * CO + n); }
    __device__ void store(int m, int n, float v) const
    {
        if (m < MT) out_[(long)m * CO + n] = v;
    }
};
using Conv2Wgrad = ConvWgrad<C1, H1, W1, C2, H2, W2, K2, S2, 128>;
using Conv3Wgrad = ConvWgrad<C2, H2, W2, C3, H3, W3, K3, S3, 64>;

// ---- conv1 weight gradient (split over frames) ---------------------------------------------------
// m = (c, kh, kw), n = o, k = (f, oy, ox); rollout frames only.
struct Conv1Wgrad : ProblemBase {
    static constexpr int BM = 256, BN = 32, BK = 16, WM = 4, WN = 1;
    static constexpr bool A_KC = false, B_KC = false;
    const uint8_t *obs;
    const float *dz1;
    float *ws;
    int M, fps;
    const uint8_t *o_;
    const float *dz_;
    float *out_;
    __device__ void bind(int agent, int split)
    {
        o_ = obs + (long)agent * M * FRAME;
        dz_ = dz1 + (long)agent * M * A1SZ;
        out_ = ws + ((long)agent * splits + split) * KW1 * C1;
        k0 = split * fps * P1;
        k1 = min(M, (split + 1) * fps) * P1;
    }
    __device__ void load_a(float (&r)[4], int m, int k) const
    {
        const int f = k / P1, p = k % P1, oy = p / W1, ox = p % W1;
        const int c = m >> 6, kh = (m >> 3) & 7, kw = m & 7;
        ld4_u8(r, o_ + (long)f * FRAME + c * (H0 * W0) + (oy * S1 + kh) * W0 + ox * S1 + kw);
    }
    __device__ void load_b(float (&r)[4], int k, int n) const { ld4(r, dz_ + (long)k * C1 + n); }
    __device__ void store(int m, int n, float v) const { out_[(long)m * C1 + n] = v; }
};

// ---- sum of split-K partials ----------------------------------------------------------------------
// out[agent][i] = sum_s part[agent][s][i]  (+ bias[i % bias_n], ReLU when bias != nullptr)
__global__ void reduce_splits_kernel(const float *__restrict__ part, int S, long len, float *out,
                                     long out_stride, const float *bias, long bias_stride, int bias_n)
{
    const int agent = blockIdx.y;
    const long i = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= len) return;
    const float *p = part + (long)agent * S * len + i;
    float4 acc = *reinterpret_cast<const float4 *>(p);
    for (int s = 1; s < S; ++s) {
        const float4 t = *reinterpret_cast<const float4 *>(p + (long)s * len);
        acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
    }
    if (bias) {
        const float *b = bias + agent * bias_stride + (i % bias_n);
        acc.x = fmaxf(acc.x + b[0], 0.f); acc.y = fmaxf(acc.y + b[1], 0.f);
        acc.z = fmaxf(acc.z + b[2], 0.f); acc.w = fmaxf(acc.w + b[3], 0.f);
    }
    *reinterpret_cast<float4 *>(out + agent * out_stride + i) = acc;
}

static hipError_t reduce_splits(const float *part, int S, long len, int N, float *out, long out_stride,
                                const float *bias, long bias_stride, int bias_n, hipStream_t s)
{
    const int blocks = (int)((len / 4 + 255) / 256);
    hipLaunchKernelGGL(reduce_splits_kernel, dim3(blocks, N), dim3(256), 0, s, part, S, len, out,
                       out_stride, bias, bias_stride, bias_n);
    return hipGetLastError();
}

// ---- column sums (bias gradients): part[agent][chunk][c] = sum over the chunk's rows --------------
template <int C>
__global__ void colsum_kernel(const float *__restrict__ in, long in_stride, int rows, int rows_per_chunk,
                              float *part)
{
    constexpr int RL = 256 / C;                     // row lanes
    __shared__ float red[256];
    const int agent = blockIdx.y, chunk = blockIdx.x;
    const int c = threadIdx.x % C, rl = threadIdx.x / C;
    const int r0 = chunk * rows_per_chunk, r1 = min(rows, r0 + rows_per_chunk);
    const float *p = in + agent * in_stride;
    float acc = 0.f;
    for (int r = r0 + rl; r < r1; r += RL) acc += p[(long)r * C + c];
    red[threadIdx.x] = acc;
    __syncthreads();
    if (rl == 0) {
        for (int j = 1; j < RL; ++j) acc += red[j * C + c];
        part[((long)agent * gridDim.x + chunk) * C + c] = acc;
    }
}

template <int C>
static hipError_t bias_grad(const float *dz, long in_stride, int rows, int N, float *ws, float *g,
                            long d_pad, long off, hipStream_t s)
{
    const int rpc = 1024;
    const int chunks = (rows + rpc - 1) / rpc;
    hipLaunchKernelGGL(colsum_kernel<C>, dim3(chunks, N), dim3(256), 0, s, dz, in_stride, rows, rpc, ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return reduce_splits(ws, chunks, C, N, g + off, d_pad, nullptr, 0, 1, s);
}

// dzh is [M][512]: one workgroup per agent, two columns per thread, frames in order.
__global__ void fc_bias_grad_kernel(const float *__restrict__ dzh, int M, float *g, long d_pad, long off)
{
    const int agent = blockIdx.x;
    const float *p = dzh + (long)agent * M * FC;
    for (int j = threadIdx.x; j < FC; j += blockDim.x) {
        float acc = 0.f;
        for (int f = 0; f < M; ++f) acc += p[(long)f * FC + j];
        g[agent * d_pad + off + j] = acc;
    }
}

// ---- heads ------------------------------------------------------------------------------------------
// One wavefront per (frame, agent): logits = W_pi h + b_pi (rollout frames), value = w_v h + b_v.
__global__ __launch_bounds__(64) void heads_fwd_kernel(const float *__restrict__ h, const float *__restrict__ x,
                                                       Layout L, int M, int F, float *logits, float *values)
{
    const int f = blockIdx.x, agent = blockIdx.y, lane = threadIdx.x;
    const float *hv = h + ((long)agent * F + f) * FC;
    const float *xa = x + agent * L.d_pad;
    float hr[FC / 64];
#pragma unroll
    for (int q = 0; q < FC / 64; ++q) hr[q] = hv[lane + 64 * q];
    const int A = L.n_actions;
    const int n_out = f < M ? A + 1 : 1;            // bootstrap states need the value only
    for (int oi = 0; oi < n_out; ++oi) {
        const bool is_v = (oi == n_out - 1);
        const float *w = is_v ? xa + L.vw : xa + L.piw + (long)oi * FC;
        float acc = 0.f;
#pragma unroll
        for (int q = 0; q < FC / 64; ++q) acc += w[lane + 64 * q] * hr[q];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (lane == 0) {
            if (is_v) values[(long)agent * F + f] = acc + xa[L.vb];
            else logits[((long)agent * M + f) * A + oi] = acc + xa[L.pib + oi];
        }
    }
}

// dzh[f][j] = (sum_a W_pi[a][j] dlogits[f][a] + w_v[j] dvalue[f]) * (h[f][j] > 0)
__global__ __launch_bounds__(256) void heads_dgrad_kernel(const float *__restrict__ h, const float *__restrict__ x,
                                                          Layout L, int M, int F, const float *__restrict__ dlogits,
                                                          const float *__restrict__ dvalues, float *dzh)
{
    const int f = blockIdx.x, agent = blockIdx.y;
    const float *xa = x + agent * L.d_pad;
    const int A = L.n_actions;
    const float *dl = dlogits + ((long)agent * M + f) * A;
    const float dv = dvalues[(long)agent * M + f];
    for (int j = threadIdx.x; j < FC; j += blockDim.x) {
        float acc = xa[L.vw + j] * dv;
        for (int a = 0; a < A; ++a) acc += xa[L.piw + (long)a * FC + j] * dl[a];
        dzh[((long)agent * M + f) * FC + j] = h[((long)agent * F + f) * FC + j] > 0.f ? acc : 0.f;
    }
}

// Head parameter gradients: row a < A of W_pi (and b_pi[a]); row A = value head.
__global__ __launch_bounds__(256) void heads_wgrad_kernel(const float *__restrict__ h, Layout L, int M, int F,
                                                          const float *__restrict__ dlogits,
                                                          const float *__restrict__ dvalues, float *g)
{
    const int row = blockIdx.x, agent = blockIdx.y;
    const int A = L.n_actions;
    const bool is_v = row == A;
    float *ga = g + agent * L.d_pad;
    const float *hv = h + (long)agent * F * FC;
    for (int j = threadIdx.x; j < FC; j += blockDim.x) {
        float acc = 0.f, sb = 0.f;
        for (int f = 0; f < M; ++f) {
            const float d = is_v ? dvalues[(long)agent * M + f] : dlogits[((long)agent * M + f) * A + row];
            acc += d * hv[(long)f * FC + j];
            sb += d;
        }
        if (is_v) ga[L.vw + j] = acc; else ga[L.piw + (long)row * FC + j] = acc;
        if (j == 0) { if (is_v) ga[L.vb] = sb; else ga[L.pib + row] = sb; }
    }
}

// ---- launch plans --------------------------------------------------------------------------------------

static inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

constexpr int FC_KCHUNK = 448;          // 3136 = 7 * 448
constexpr int FPS_CONV1 = 2, FPS_CONV2 = 8, FPS_CONV3 = 16;   // frames per split of the weight gradients

size_t workspace_floats(int N, int M, int F)
{
    size_t need = (size_t)N * cdiv(FLAT, FC_KCHUNK) * F * FC;
    auto mx = [&](size_t v) { if (v > need) need = v; };
    mx((size_t)N * cdiv(M, FPS_CONV1) * KW1 * C1);
    mx((size_t)N * cdiv(M, FPS_CONV2) * KW2 * C2);
    mx((size_t)N * cdiv(M, FPS_CONV3) * KW3 * C3);
    mx((size_t)N * cdiv((long)M * P1, 1024) * C1);
    return need + 1024;
}

#define GALA_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return e_; } while (0)

hipError_t launch_forward(const NetArgs &a, hipStream_t s, PhaseTimer *pt)
{
    const Layout &L = a.L;
    {
        Conv1Fwd p{};
        p.obs = a.obs; p.boot = a.boot; p.x = a.x; p.a1 = a.b.a1; p.d_pad = L.d_pad; p.w_off = L.w1; p.b_off = L.b1;
        p.M = a.M; p.F = a.F; p.Bn = a.Bn;
        p.tiles_m = cdiv((long)a.F * P1, Conv1Fwd::BM); p.tiles_n = 1; p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("conv1_fwd");
    }
    {
        Conv2Fwd p{};
        p.in = a.b.a1; p.x = a.x; p.out = a.b.a2; p.d_pad = L.d_pad; p.w_off = L.w2; p.b_off = L.b2; p.F = a.F;
        p.tiles_m = cdiv((long)a.F * P2, Conv2Fwd::BM); p.tiles_n = 1; p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("conv2_fwd");
    }
    {
        Conv3Fwd p{};
        p.in = a.b.a2; p.x = a.x; p.out = a.b.a3; p.d_pad = L.d_pad; p.w_off = L.w3; p.b_off = L.b3; p.F = a.F;
        p.tiles_m = cdiv((long)a.F * P3, Conv3Fwd::BM); p.tiles_n = 1; p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("conv3_fwd");
    }
    {
        FcFwd p{};
        p.a3 = a.b.a3; p.x = a.x; p.ws = a.b.ws; p.d_pad = L.d_pad; p.w_off = L.fcw; p.F = a.F;
        p.kchunk = FC_KCHUNK;
        p.tiles_m = cdiv(a.F, FcFwd::BM); p.tiles_n = FC / FcFwd::BN; p.splits = cdiv(FLAT, FC_KCHUNK);
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("fc_fwd");
        GALA_TRY(reduce_splits(a.b.ws, p.splits, (long)a.F * FC, a.N, a.b.h, (long)a.F * FC,
                               a.x + L.fcb, L.d_pad, FC, s));
        pt->mark("fc_fwd_reduce");
    }
    hipLaunchKernelGGL(heads_fwd_kernel, dim3(a.F, a.N), dim3(64), 0, s, a.b.h, a.x, L, a.M, a.F,
                       a.b.logits, a.b.values);
    pt->mark("heads_fwd");
    return hipGetLastError();
}

hipError_t launch_backward(const NetArgs &a, hipStream_t s, PhaseTimer *pt)
{
    const Layout &L = a.L;
    hipLaunchKernelGGL(heads_dgrad_kernel, dim3(a.M, a.N), dim3(256), 0, s, a.b.h, a.x, L, a.M, a.F,
                       a.b.dlogits, a.b.dvalues, a.b.dzh);
    GALA_TRY(hipGetLastError());
    pt->mark("heads_dgrad");
    hipLaunchKernelGGL(heads_wgrad_kernel, dim3(L.n_actions + 1, a.N), dim3(256), 0, s, a.b.h, L, a.M, a.F,
                       a.b.dlogits, a.b.dvalues, a.b.g);
    GALA_TRY(hipGetLastError());
    pt->mark("heads_wgrad");
    hipLaunchKernelGGL(fc_bias_grad_kernel, dim3(a.N), dim3(256), 0, s, a.b.dzh, a.M, a.b.g, L.d_pad, L.fcb);
    GALA_TRY(hipGetLastError());
    pt->mark("fc_bgrad");
    {
        FcWgrad p{};
        p.dzh = a.b.dzh; p.a3 = a.b.a3; p.g = a.b.g; p.d_pad = L.d_pad; p.w_off = L.fcw; p.M = a.M; p.F = a.F;
        p.tiles_m = FC / FcWgrad::BM; p.tiles_n = cdiv(FLAT, FcWgrad::BN); p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("fc_wgrad");
    }
    {
        FcDgrad p{};
        p.dzh = a.b.dzh; p.x = a.x; p.a3 = a.b.a3; p.dz3 = a.b.dz3; p.d_pad = L.d_pad; p.w_off = L.fcw;
        p.M = a.M; p.F = a.F;
        p.tiles_m = cdiv(a.M, FcDgrad::BM); p.tiles_n = cdiv(FLAT, FcDgrad::BN); p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("fc_dgrad");
    }
    // conv3
    GALA_TRY(bias_grad<C3>(a.b.dz3, (long)a.M * A3SZ, a.M * P3, a.N, a.b.ws, a.b.g, L.d_pad, L.b3, s));
    pt->mark("conv3_bgrad");
    {
        Conv3Wgrad p{};
        p.in = a.b.a2; p.dz = a.b.dz3; p.ws = a.b.ws; p.M = a.M; p.F = a.F; p.fps = FPS_CONV3;
        p.tiles_m = cdiv(KW3, Conv3Wgrad::BM); p.tiles_n = 1; p.splits = cdiv(a.M, FPS_CONV3);
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("conv3_wgrad");
        GALA_TRY(reduce_splits(a.b.ws, p.splits, (long)KW3 * C3, a.N, a.b.g + L.w3, L.d_pad, nullptr, 0, 1, s));
        pt->mark("conv3_wgrad_reduce");
    }
    {
        Conv3Dgrad p{};
        p.dz3 = a.b.dz3; p.x = a.x; p.a2 = a.b.a2; p.dz2 = a.b.dz2; p.d_pad = L.d_pad; p.w_off = L.w3;
        p.M = a.M; p.F = a.F;
        p.tiles_m = cdiv((long)a.M * P2, Conv3Dgrad::BM); p.tiles_n = 1; p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("conv3_dgrad");
    }
    // conv2
    GALA_TRY(bias_grad<C2>(a.b.dz2, (long)a.M * A2SZ, a.M * P2, a.N, a.b.ws, a.b.g, L.d_pad, L.b2, s));
    pt->mark("conv2_bgrad");
    {
        Conv2Wgrad p{};
        p.in = a.b.a1; p.dz = a.b.dz2; p.ws = a.b.ws; p.M = a.M; p.F = a.F; p.fps = FPS_CONV2;
        p.tiles_m = cdiv(KW2, Conv2Wgrad::BM); p.tiles_n = 1; p.splits = cdiv(a.M, FPS_CONV2);
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("conv2_wgrad");
        GALA_TRY(reduce_splits(a.b.ws, p.splits, (long)KW2 * C2, a.N, a.b.g + L.w2, L.d_pad, nullptr, 0, 1, s));
        pt->mark("conv2_wgrad_reduce");
    }
    {
        Conv2Dgrad p{};
        p.dz2 = a.b.dz2; p.x = a.x; p.a1 = a.b.a1; p.dz1 = a.b.dz1; p.d_pad = L.d_pad; p.w_off = L.w2;
        p.M = a.M; p.F = a.F;
        p.tiles_m = cdiv((long)a.M * Conv2Dgrad::PC, Conv2Dgrad::BM); p.tiles_n = 1; p.splits = 4;
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("conv2_dgrad");
    }
    // conv1 (the input needs no gradient)
    GALA_TRY(bias_grad<C1>(a.b.dz1, (long)a.M * A1SZ, a.M * P1, a.N, a.b.ws, a.b.g, L.d_pad, L.b1, s));
    pt->mark("conv1_bgrad");
    {
        Conv1Wgrad p{};
        p.obs = a.obs; p.dz1 = a.b.dz1; p.ws = a.b.ws; p.M = a.M; p.fps = FPS_CONV1;
        p.tiles_m = 1; p.tiles_n = 1; p.splits = cdiv(a.M, FPS_CONV1);
        GALA_TRY(igemm_launch(p, a.N, s));
        pt->mark("conv1_wgrad");
        GALA_TRY(reduce_splits(a.b.ws, p.splits, (long)KW1 * C1, a.N, a.b.g + L.w1, L.d_pad, nullptr, 0, 1, s));
        pt->mark("conv1_wgrad_reduce");
    }
    return hipSuccess;
}

}  // namespace gala
