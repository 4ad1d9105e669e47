// Diagnostics of Sec. 5 "Effects of gossip": the pair-wise cosine similarity of the agents'
// gradients (Fig. 2b) as a Gram matrix on the matrix cores, and the size of a round's local
// updates ||alpha G|| that enters the bound of Prop. 1.
#include "gala_internal.h"

namespace gala {

typedef float diag_f32x4 __attribute__((ext_vector_type(4)));

// ---- Gram matrix  G G^T  of the gradient arena ------------------------------------------------
// Agents are cut into tiles of GRAM_T rows; a workgroup owns one pair of tiles (ti <= tj) and
// one contiguous range of parameter columns, which its four wavefronts walk in steps of 16
// columns, GRAM_UNROLL consecutive steps per wavefront at a time (256 contiguous bytes of every
// row, so that both halves of a cache line are asked for by the same wavefront back to back).
// No LDS staging is needed: lane l loads the float4 of agent l % 16 at columns
// 4 (l / 16) .. + 3 of the step, and element e of that float4 is the lane's operand of
// the e-th 16x16x4 fp32 MFMA.  That pairs the MFMA's k index (l / 16) with column
// 4 (l / 16) + e, a permutation of the step's 16 columns that is the same for both operands,
// which is all a sum over columns needs.  The wavefronts' results are added in a fixed order
// and stored per (pair, chunk).  Every gradient is read once per tile pair it takes part in:
// the kernel is bound by HBM.
constexpr int GRAM_STEP = 16;           // columns per MFMA group
constexpr int GRAM_UNROLL = 4;          // steps in flight per wavefront
constexpr int GRAM_WORKGROUPS = 256;    // workgroups in all (more, or more steps in flight, change nothing: measured)

__global__ __launch_bounds__(256) void gram_kernel(const float *__restrict__ g, int N, long d_pad, int tiles,
                                                   int chunks, float *__restrict__ part)
{
    __shared__ float red[4 * GRAM_T * GRAM_T];
    // pair index -> (ti, tj), ti <= tj
    int ti = 0, rest = blockIdx.y;
    while (rest >= tiles - ti) { rest -= tiles - ti; ++ti; }
    const int tj = ti + rest;
    const bool same = ti == tj;
    const int chunk = blockIdx.x;
    const long steps = d_pad / GRAM_STEP;
    const long per = (steps + chunks - 1) / chunks;
    const long s0 = chunk * per, s1 = s0 + per < steps ? s0 + per : steps;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;

    diag_f32x4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = diag_f32x4{0.f, 0.f, 0.f, 0.f};

    // this lane's two agents per tile; rows beyond the last agent are read as zero from row 0
    const int ra0 = ti * GRAM_T + lr, ra1 = ra0 + 16, rb0 = tj * GRAM_T + lr, rb1 = rb0 + 16;
    const bool va0 = ra0 < N, va1 = ra1 < N, vb0 = rb0 < N, vb1 = rb1 < N;
    const float *pa0 = g + (va0 ? (long)ra0 * d_pad : 0L) + 4 * lk, *pa1 = g + (va1 ? (long)ra1 * d_pad : 0L) + 4 * lk;
    const float *pb0 = g + (vb0 ? (long)rb0 * d_pad : 0L) + 4 * lk, *pb1 = g + (vb1 ? (long)rb1 * d_pad : 0L) + 4 * lk;
    auto ld = [&](const float *p, bool valid, long ss) -> float4 {
        float4 v = *reinterpret_cast<const float4 *>(p + (ss < s1 ? ss : s0) * GRAM_STEP);   // always in range
        if (!(valid && ss < s1)) v = make_float4(0.f, 0.f, 0.f, 0.f);
        return v;
    };
    auto mma4 = [&](const float4 &x0, const float4 &x1, const float4 &y0, const float4 &y1) {
        const float xa[4] = {x0.x, x0.y, x0.z, x0.w}, xb[4] = {x1.x, x1.y, x1.z, x1.w};
        const float ya[4] = {y0.x, y0.y, y0.z, y0.w}, yb[4] = {y1.x, y1.y, y1.z, y1.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[e], ya[e], acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[e], yb[e], acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(xb[e], ya[e], acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(xb[e], yb[e], acc[1][1], 0, 0, 0);
        }
    };
    if (same) {
        constexpr int U = GRAM_UNROLL;
        for (long s = s0 + wave * U; s < s1; s += 4 * U) {
            float4 a0[U], a1[U];
#pragma unroll
            for (int u = 0; u < U; ++u) { a0[u] = ld(pa0, va0, s + u); a1[u] = ld(pa1, va1, s + u); }
#pragma unroll
            for (int u = 0; u < U; ++u) mma4(a0[u], a1[u], a0[u], a1[u]);
        }
    } else {
        for (long s = s0 + wave * GRAM_UNROLL; s < s1; s += 4 * GRAM_UNROLL) {
            float4 a0[GRAM_UNROLL], a1[GRAM_UNROLL], b0[GRAM_UNROLL], b1[GRAM_UNROLL];
#pragma unroll
            for (int u = 0; u < GRAM_UNROLL; ++u) {
                a0[u] = ld(pa0, va0, s + u); a1[u] = ld(pa1, va1, s + u);
                b0[u] = ld(pb0, vb0, s + u); b1[u] = ld(pb1, vb1, s + u);
            }
#pragma unroll
            for (int u = 0; u < GRAM_UNROLL; ++u) mma4(a0[u], a1[u], b0[u], b1[u]);
        }
    }
    // accumulator register v of lane l holds row 4 * (l / 16) + v, column l % 16 of its block
    static_assert(GRAM_T == 32, "two 16-row blocks per tile side");
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                red[wave * (GRAM_T * GRAM_T) + (i * 16 + 4 * lk + v) * GRAM_T + j * 16 + lr] = acc[i][j][v];
    __syncthreads();
    float *out = part + ((long)blockIdx.y * chunks + chunk) * (GRAM_T * GRAM_T);
    for (int e = tid; e < GRAM_T * GRAM_T; e += 256)
        out[e] = (red[e] + red[GRAM_T * GRAM_T + e]) + (red[2 * GRAM_T * GRAM_T + e] + red[3 * GRAM_T * GRAM_T + e]);
}

// Sum the chunks of a tile pair and scatter the tile (and its mirror image) into gram [N][N].
// One workgroup per (pair, tile row): 32 elements, 32 threads each over interleaved chunks (four
// chains per thread), combined in thread order.
__global__ __launch_bounds__(1024) void gram_reduce_kernel(const float *__restrict__ part, int N, int tiles,
                                                           int chunks, float *gram)
{
    __shared__ float red[32][GRAM_T];
    int ti = 0, rest = blockIdx.x;
    while (rest >= tiles - ti) { rest -= tiles - ti; ++ti; }
    const int tj = ti + rest;
    const int r = blockIdx.y, c = threadIdx.x % GRAM_T, q = threadIdx.x / GRAM_T;
    const float *p = part + (long)blockIdx.x * chunks * (GRAM_T * GRAM_T) + r * GRAM_T + c;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    int k = q;
    for (; k + 96 < chunks; k += 128) {
        a0 += p[(long)k * (GRAM_T * GRAM_T)];
        a1 += p[(long)(k + 32) * (GRAM_T * GRAM_T)];
        a2 += p[(long)(k + 64) * (GRAM_T * GRAM_T)];
        a3 += p[(long)(k + 96) * (GRAM_T * GRAM_T)];
    }
    for (; k < chunks; k += 32) a0 += p[(long)k * (GRAM_T * GRAM_T)];
    red[q][c] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (q == 0) {
        float t = 0.f;
        for (int w = 0; w < 32; ++w) t += red[w][c];
        const int i = ti * GRAM_T + r, j = tj * GRAM_T + c;
        if (i < N && j < N) {
            gram[(long)i * N + j] = t;
            if (ti != tj) gram[(long)j * N + i] = t;
        }
    }
}

// cos_ij = <g_i, g_j> / (||g_i|| ||g_j||), 0 where a gradient is zero
__global__ __launch_bounds__(256) void cosine_kernel(const float *__restrict__ gram, int N, float *cosm)
{
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    if (e >= (long)N * N) return;
    const int i = (int)(e / N), j = (int)(e % N);
    const float ni = sqrtf(gram[(long)i * N + i]), nj = sqrtf(gram[(long)j * N + j]);
    cosm[e] = (ni > 0.f && nj > 0.f) ? gram[e] / (ni * nj) : 0.f;
}

int gram_tiles(int N) { return (N + GRAM_T - 1) / GRAM_T; }
int gram_pairs(int N) { const int t = gram_tiles(N); return t * (t + 1) / 2; }
int gram_chunks(int N)
{
    int c = GRAM_WORKGROUPS / gram_pairs(N);
    return c < 1 ? 1 : c;
}

hipError_t launch_grad_cosine(int N, const Layout &L, const float *g, float *part, float *gram, float *cosm,
                              hipStream_t s)
{
    const int tiles = gram_tiles(N), pairs = gram_pairs(N), chunks = gram_chunks(N);
    hipLaunchKernelGGL(gram_kernel, dim3(chunks, pairs), dim3(256), 0, s, g, N, L.d_pad, tiles, chunks, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gram_reduce_kernel, dim3(pairs, GRAM_T), dim3(1024), 0, s, part, N, tiles, chunks, gram);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(cosine_kernel, dim3((unsigned)(((long)N * N + 255) / 256)), dim3(256), 0, s, gram, N, cosm);
    return hipGetLastError();
}

// ---- size of the last optimiser step (Prop. 1: the update matrix alpha G) --------------------------
// RMSprop moved agent i by  lr c_i g / (sqrt(v) + eps)  with the already updated v; the sum of
// its squares is rebuilt from the gradient and the optimizer state, no copy of the old
// parameters is needed.  g_stride = 0 when all agents applied the same (averaged) gradient.
__global__ __launch_bounds__(256) void update_sumsq_kernel(const float *__restrict__ g, long g_stride,
                                                           const float *__restrict__ v, long d_pad,
                                                           const float *__restrict__ stats, float lr, float eps,
                                                           float *part)
{
    __shared__ float red[4];
    const int agent = blockIdx.y;
    const float c = stats[agent * 5 + 4];
    const float4 *g4 = reinterpret_cast<const float4 *>(g + agent * g_stride);
    const float4 *v4 = reinterpret_cast<const float4 *>(v + agent * d_pad);
    float acc = 0.f;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < d_pad / 4; i += (long)gridDim.x * 256) {
        const float4 gg = g4[i], vv = v4[i];
        const float a = lr * (c * gg.x) / (sqrtf(vv.x) + eps), b = lr * (c * gg.y) / (sqrtf(vv.y) + eps);
        const float p = lr * (c * gg.z) / (sqrtf(vv.z) + eps), q = lr * (c * gg.w) / (sqrtf(vv.w) + eps);
        acc += (a * a + b * b) + (p * p + q * q);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) part[agent * UPDATE_NORM_BLOCKS + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// out[i] = ||alpha g_i||_2 for i < N, out[N] = largest of them, out[N + 1] = ||alpha G||_F
hipError_t launch_update_norm(int N, const Layout &L, const HParams &hp, const float *g, bool shared_gradient,
                              const float *v, const float *stats, float *part, float *row_ss, float *out,
                              hipStream_t s)
{
    hipLaunchKernelGGL(update_sumsq_kernel, dim3(UPDATE_NORM_BLOCKS, N), dim3(256), 0, s, g,
                       shared_gradient ? 0L : L.d_pad, v, L.d_pad, stats, hp.lr, hp.rms_eps, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_row_norms(part, N, UPDATE_NORM_BLOCKS, row_ss, out, out + N, s);
}

}  // namespace gala
