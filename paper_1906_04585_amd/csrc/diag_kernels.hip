// Diagnostics of Sec. 5 "Effects of gossip": the pair-wise cosine similarity of the agents'
// gradients (Fig. 2b) as a Gram matrix on the matrix cores, and the size of a round's local
// updates ||alpha G|| that enters the bound of Prop. 1.
#include "gala_internal.h"

namespace gala {

typedef float diag_f32x4 __attribute__((ext_vector_type(4)));

// ---- Gram matrix  G G^T  of the gradient arena ------------------------------------------------
// Agents are cut into tiles of GRAM_T rows; a workgroup owns one pair of tiles (ti <= tj) and one
// contiguous range of parameter columns, which it walks GRAM_COLS columns at a time.  Memory is read
// the way it is laid out: every wavefront load takes one KB of one agent's row (lane l the float4
// at columns 4 l), eight rows per wavefront and tile side; the next slab's loads are in flight while
// the current one is multiplied.  The slab goes to LDS ([row][GRAM_COLS + 4]: the four floats of
// padding put the sixteen rows of an operand read on sixteen groups of four banks), from where a
// wavefront reads its own 64 columns as MFMA operands: lane l takes the float4 of agent l % 16 at
// columns 4 (l / 16) .. + 3 of a 16-column step, and element e of that float4 is the lane's operand
// of the e-th 16x16x4 fp32 MFMA.  That pairs the MFMA's k index (l / 16) with column 4 (l / 16) + e,
// a permutation of the step's 16 columns that is the same for both operands, which is all a sum
// over columns needs.  On the diagonal (ti == tj) the lower left block is the transpose of the upper
// right one and is not computed.  The wavefronts' results are added in a fixed order and stored per
// (pair, chunk).  Every gradient is read once per tile pair it takes part in: the kernel is bound by
// HBM (loading the operands from global memory straight into the MFMA lanes, 64 bytes per row and
// load, ran at 3.0 TB/s; this form reads whole lines).
constexpr int GRAM_STEP = 16;           // columns per MFMA group
constexpr int GRAM_COLS = 256;          // columns per slab: one KB per row
constexpr int GRAM_PITCH = GRAM_COLS + 4;
constexpr int GRAM_WORKGROUPS = 1024;   // workgroups in all

template <bool SAME>
__device__ __forceinline__ void gram_body(const float *__restrict__ g, int N, long d_pad, int ti, int tj,
                                          long t0, long t1, float *smem, diag_f32x4 (&acc)[2][2])
{
    constexpr int SIDES = SAME ? 1 : 2;
    constexpr int NL = 8 * SIDES;                       // float4 loads per thread and slab
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;
    // rows this thread loads: 8 per side, rows of a missing agent are read from row 0 and zeroed
    const float *src[NL];
    bool valid[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int r = (i < 8 ? ti : tj) * GRAM_T + wave * 8 + (i & 7);
        valid[i] = r < N;
        src[i] = g + (valid[i] ? (long)r * d_pad : 0L) + 4 * lane;
    }
    float4 regs[NL];
    auto fetch = [&](long t) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {        // read once, whole lines: the non-temporal hint (70 -> 42 us from HBM)
            const diag_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const diag_f32x4 *>(src[i] + t * GRAM_COLS));
            regs[i] = make_float4(v[0], v[1], v[2], v[3]);
        }
    };
    auto lds_row = [&](int side, int row) { return smem + (side * GRAM_T + row) * GRAM_PITCH; };
    if (t0 < t1) fetch(t0);
    for (long t = t0; t < t1; ++t) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const float4 v = valid[i] ? regs[i] : make_float4(0.f, 0.f, 0.f, 0.f);
            *reinterpret_cast<float4 *>(lds_row(i >> 3, wave * 8 + (i & 7)) + 4 * lane) = v;
        }
        __syncthreads();
        if (t + 1 < t1) fetch(t + 1);
#pragma unroll
        for (int st = 0; st < GRAM_COLS / 4 / GRAM_STEP; ++st) {
            const int col = wave * (GRAM_COLS / 4) + st * GRAM_STEP + 4 * lk;
            const float4 x0 = *reinterpret_cast<const float4 *>(lds_row(0, lr) + col);
            const float4 x1 = *reinterpret_cast<const float4 *>(lds_row(0, lr + 16) + col);
            const float4 y0 = SAME ? x0 : *reinterpret_cast<const float4 *>(lds_row(1, lr) + col);
            const float4 y1 = SAME ? x1 : *reinterpret_cast<const float4 *>(lds_row(1, lr + 16) + col);
            const float xa[4] = {x0.x, x0.y, x0.z, x0.w}, xb[4] = {x1.x, x1.y, x1.z, x1.w};
            const float ya[4] = {y0.x, y0.y, y0.z, y0.w}, yb[4] = {y1.x, y1.y, y1.z, y1.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[e], ya[e], acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[e], yb[e], acc[0][1], 0, 0, 0);
                if (!SAME) acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(xb[e], ya[e], acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(xb[e], yb[e], acc[1][1], 0, 0, 0);
            }
        }
        __syncthreads();
    }
}

// SIDES = 1: a single tile of agents (N <= GRAM_T), half the LDS
template <int SIDES>
__global__ __launch_bounds__(256) void gram_kernel(const float *__restrict__ g, int N, long d_pad, int tiles,
                                                   int chunks, float *__restrict__ part)
{
    __shared__ __attribute__((aligned(16))) float smem[SIDES * GRAM_T * GRAM_PITCH];
    static_assert(GRAM_T * GRAM_PITCH >= 4 * GRAM_T * GRAM_T, "the slab also holds the wavefronts' results");
    // pair index -> (ti, tj), ti <= tj
    int ti = 0, rest = blockIdx.y;
    while (rest >= tiles - ti) { rest -= tiles - ti; ++ti; }
    const int tj = ti + rest;
    const bool same = ti == tj;
    const int chunk = blockIdx.x;
    const long slabs = d_pad / GRAM_COLS;               // the arena's row length is a multiple of GRAM_COLS
    const long per = (slabs + chunks - 1) / chunks;
    const long t0 = chunk * per, t1 = t0 + per < slabs ? t0 + per : slabs;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;

    diag_f32x4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = diag_f32x4{0.f, 0.f, 0.f, 0.f};
    if (SIDES == 1 || same) gram_body<true>(g, N, d_pad, ti, tj, t0, t1, smem, acc);
    else if constexpr (SIDES == 2) gram_body<false>(g, N, d_pad, ti, tj, t0, t1, smem, acc);

    // accumulator register v of lane l holds row 4 * (l / 16) + v, column l % 16 of its block
    static_assert(GRAM_T == 32, "two 16-row blocks per tile side");
    float *red = smem;                                   // the loop ended with a barrier
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (same && i == 1 && j == 0)            // mirror image of the upper right block
                    red[wave * (GRAM_T * GRAM_T) + (16 + lr) * GRAM_T + 4 * lk + v] = acc[0][1][v];
                else
                    red[wave * (GRAM_T * GRAM_T) + (i * 16 + 4 * lk + v) * GRAM_T + j * 16 + lr] = acc[i][j][v];
            }
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
static_assert(GRAM_WORKGROUPS >= 1, "at least one chunk");

hipError_t launch_grad_cosine(int N, const Layout &L, const float *g, float *part, float *gram, float *cosm,
                              hipStream_t s)
{
    const int tiles = gram_tiles(N), pairs = gram_pairs(N), chunks = gram_chunks(N);
    if (L.d_pad % GRAM_COLS != 0) return hipErrorInvalidValue;      // the layout pads every agent's slice to whole KB
    if (tiles == 1) hipLaunchKernelGGL(gram_kernel<1>, dim3(chunks, pairs), dim3(256), 0, s, g, N, L.d_pad, tiles, chunks, part);
    else hipLaunchKernelGGL(gram_kernel<2>, dim3(chunks, pairs), dim3(256), 0, s, g, N, L.d_pad, tiles, chunks, part);
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
        // both arenas are read once: non-temporal (81 -> 73 us, and the parameters stay cached for what follows)
        const diag_f32x4 gn = __builtin_nontemporal_load(reinterpret_cast<const diag_f32x4 *>(g4 + i));
        const diag_f32x4 vn = __builtin_nontemporal_load(reinterpret_cast<const diag_f32x4 *>(v4 + i));
        const float4 gg = make_float4(gn[0], gn[1], gn[2], gn[3]), vv = make_float4(vn[0], vn[1], vn[2], vn[3]);
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
