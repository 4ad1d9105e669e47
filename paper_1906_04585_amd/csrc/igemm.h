// Agent-grouped implicit-GEMM on the gfx950 matrix cores (fp32 MFMA 32x32x2).
//
// One launch computes, for every agent, C[m][n] = sum_k A[m][k] * B[k][n] where A and
// B are *views* described by a problem functor P (im2col of an activation tensor, a
// weight matrix, a byte image, ...) and C is consumed element-wise by P::store.  The
// kernel never materialises A or B in HBM: 256 threads stage BM x BK and BK x BN tiles
// through LDS (k-major, so a wavefront's MFMA operand read is one conflict-free
// ds_read_b32 per lane), double-buffered against the global loads of the next k-tile.
//
// P provides
//   static constexpr int  BM, BN, BK        tile sizes (BK multiple of 4)
//   static constexpr int  WM, WN            wavefront grid, WM*WN == 4; each wavefront
//                                           owns (BM/WM) x (BN/WN), multiples of 32
//   static constexpr bool A_KC, B_KC        true: the operand is read in groups of 4
//                                           consecutive k; false: 4 consecutive m (or n)
//   int tiles_m, tiles_n, splits            filled by the host
//   void bind(int agent, int split)         per-agent pointers and the split's k-range
//   int  k_begin(), k_end()
//   void load_a(float (&r)[4], int m, int k)   zero-fills outside the problem
//   void load_b(float (&r)[4], int k, int n)
//   void store(int m, int n, float v)
//
// Workgroup ids are interleaved over the 8 XCDs by the dispatcher; the decode below
// keeps all tiles of one agent on one XCD so that its weights and activations are
// shared through that XCD's L2.
#pragma once
#include <hip/hip_runtime.h>

typedef float gala_f32x16 __attribute__((ext_vector_type(16)));

template <class P>
__global__ __launch_bounds__(256) void igemm_kernel(P p, int n_agents)
{
    constexpr int BM = P::BM, BN = P::BN, BK = P::BK;
    constexpr int PAD = 4;
    constexpr int SA = BM + PAD, SB = BN + PAD;
    constexpr int WTM = BM / P::WM, WTN = BN / P::WN;   // wavefront tile
    constexpr int BI = WTM / 32, BJ = WTN / 32;
    static_assert(P::WM * P::WN == 4, "four wavefronts per workgroup");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wavefront tile in 32x32 blocks");
    static_assert(BK % 4 == 0 && BM % 4 == 0 && BN % 4 == 0, "vector groups of four");

    __shared__ __attribute__((aligned(16))) float As[2][BK][SA];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK][SB];

    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int tiles = p.tiles_m * p.tiles_n * p.splits;
    const int agent = (slot / tiles) * 8 + xcd;
    if (agent >= n_agents) return;
    int tile = slot % tiles;
    const int tn = tile % p.tiles_n; tile /= p.tiles_n;
    const int tm = tile % p.tiles_m; tile /= p.tiles_m;
    const int split = tile;
    p.bind(agent, split);
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / P::WN) * WTM, wn0 = (wave % P::WN) * WTN;

    constexpr int GA = BM * BK / 4, GB = BN * BK / 4;       // groups of four per tile
    constexpr int PA = (GA + 255) / 256, PB = (GB + 255) / 256;
    float ra[PA][4], rb[PB][4];

    const int kb = p.k_begin(), ke = p.k_end();

    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const int g = tid + i * 256;
            ra[i][0] = ra[i][1] = ra[i][2] = ra[i][3] = 0.f;
            if (GA % 256 == 0 || g < GA) {
                if (P::A_KC) {
                    const int row = g / (BK / 4), kq = g % (BK / 4);
                    if (k0 + kq * 4 < ke) p.load_a(ra[i], m0 + row, k0 + kq * 4);
                } else {
                    const int k = g / (BM / 4), mq = g % (BM / 4);
                    if (k0 + k < ke) p.load_a(ra[i], m0 + mq * 4, k0 + k);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            const int g = tid + i * 256;
            rb[i][0] = rb[i][1] = rb[i][2] = rb[i][3] = 0.f;
            if (GB % 256 == 0 || g < GB) {
                if (P::B_KC) {
                    const int col = g / (BK / 4), kq = g % (BK / 4);
                    if (k0 + kq * 4 < ke) p.load_b(rb[i], k0 + kq * 4, n0 + col);
                } else {
                    const int k = g / (BN / 4), nq = g % (BN / 4);
                    if (k0 + k < ke) p.load_b(rb[i], k0 + k, n0 + nq * 4);
                }
            }
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const int g = tid + i * 256;
            if (GA % 256 == 0 || g < GA) {
                if (P::A_KC) {
                    const int row = g / (BK / 4), kq = g % (BK / 4);
#pragma unroll
                    for (int j = 0; j < 4; ++j) As[buf][kq * 4 + j][row] = ra[i][j];
                } else {
                    const int k = g / (BM / 4), mq = g % (BM / 4);
                    *reinterpret_cast<float4 *>(&As[buf][k][mq * 4]) =
                        make_float4(ra[i][0], ra[i][1], ra[i][2], ra[i][3]);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            const int g = tid + i * 256;
            if (GB % 256 == 0 || g < GB) {
                if (P::B_KC) {
                    const int col = g / (BK / 4), kq = g % (BK / 4);
#pragma unroll
                    for (int j = 0; j < 4; ++j) Bs[buf][kq * 4 + j][col] = rb[i][j];
                } else {
                    const int k = g / (BN / 4), nq = g % (BN / 4);
                    *reinterpret_cast<float4 *>(&Bs[buf][k][nq * 4]) =
                        make_float4(rb[i][0], rb[i][1], rb[i][2], rb[i][3]);
                }
            }
        }
    };

    gala_f32x16 acc[BI][BJ];
#pragma unroll
    for (int i = 0; i < BI; ++i)
#pragma unroll
        for (int j = 0; j < BJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nkt = (ke - kb + BK - 1) / BK;
    if (nkt > 0) {
        fetch(kb);
        stage(0);
    }
    __syncthreads();
    const int lr = lane & 31, lk = lane >> 5;
    for (int kt = 0; kt < nkt; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nkt) fetch(kb + (kt + 1) * BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float a[BI], b[BJ];
#pragma unroll
            for (int i = 0; i < BI; ++i) a[i] = As[buf][kk + lk][wm0 + i * 32 + lr];
#pragma unroll
            for (int j = 0; j < BJ; ++j) b[j] = Bs[buf][kk + lk][wn0 + j * 32 + lr];
#pragma unroll
            for (int i = 0; i < BI; ++i)
#pragma unroll
                for (int j = 0; j < BJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nkt) stage(buf ^ 1);
        __syncthreads();
    }

    // D layout of the 32x32 MFMA: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4,
    // column l%32.
#pragma unroll
    for (int i = 0; i < BI; ++i)
#pragma unroll
        for (int j = 0; j < BJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm0 + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
                const int n = n0 + wn0 + j * 32 + lr;
                p.store(m, n, acc[i][j][v]);
            }
}

template <class P>
static inline hipError_t igemm_launch(const P &p, int n_agents, hipStream_t stream)
{
    const int agents_pad = (n_agents + 7) / 8 * 8;
    const int grid = agents_pad * p.tiles_m * p.tiles_n * p.splits;
    hipLaunchKernelGGL(igemm_kernel<P>, dim3(grid), dim3(256), 0, stream, p, n_agents);
    return hipGetLastError();
}
