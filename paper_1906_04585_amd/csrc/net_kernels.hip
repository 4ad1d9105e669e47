// Agent-grouped forward and backward passes of the 3-conv / 1-hidden / two-head network
// (App. C.2 of the paper) as implicit GEMMs on the fp32 matrix cores, plus the small
// kernels around them (heads, bias gradients, split-K reduction).
//
// Activations are channels-last: a1 [f][20][20][32], a2 [f][9][9][64], a3 [f][7][7][64],
// h [f][512]; frame f < M is rollout sample t*B + b, frames M..F-1 are the bootstrap
// states.  Backward buffers hold gradients w.r.t. the values *before* each ReLU.
#include "gala_internal.h"
#include "igemm.h"

#ifndef GALA_MFMA16
#define GALA_MFMA16 true
#endif

namespace gala {

// Loads by (uniform base pointer, per-lane byte offset): the base stays in scalar registers.
static __device__ __forceinline__ float4 ldg4b(const void *base, unsigned boff)
{
    return *reinterpret_cast<const float4 *>(static_cast<const char *>(base) + boff);
}
// Streams that nothing reads again soon (the hidden layer's weights in its data gradient, its weight gradient on
// the way out) carry the non-temporal hint, so that they do not push out what the next kernels read.
typedef float stream_f32x4 __attribute__((ext_vector_type(4)));
static __device__ __forceinline__ float4 ldg4b_stream(const void *base, unsigned boff)
{
    const stream_f32x4 t =
        __builtin_nontemporal_load(reinterpret_cast<const stream_f32x4 *>(static_cast<const char *>(base) + boff));
    return make_float4(t.x, t.y, t.z, t.w);
}
static __device__ __forceinline__ void st4_stream(float *p, float4 v)
{
    const stream_f32x4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<stream_f32x4 *>(p));
}
static __device__ __forceinline__ uint32_t ldg_u32b(const void *base, unsigned boff)
{
    return *reinterpret_cast<const uint32_t *>(static_cast<const char *>(base) + boff);
}
static __device__ __forceinline__ float4 relu_bias4(float4 v, float4 b)
{
    return make_float4(fmaxf(v.x + b.x, 0.f), fmaxf(v.y + b.y, 0.f), fmaxf(v.z + b.z, 0.f), fmaxf(v.w + b.w, 0.f));
}
// gradient passes where the forward activation was positive
static __device__ __forceinline__ float4 relu_mask4(float4 v, float4 act)
{
    return make_float4(act.x > 0.f ? v.x : 0.f, act.y > 0.f ? v.y : 0.f, act.z > 0.f ? v.z : 0.f,
                       act.w > 0.f ? v.w : 0.f);
}
static __device__ __forceinline__ float4 scale4(float4 v, float s) { return make_float4(v.x * s, v.y * s, v.z * s, v.w * s); }
static __device__ __forceinline__ void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
static __device__ __forceinline__ void unpack(float (&r)[4], float4 v)
{
    r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
}
// Four state bytes as floats 0..255.  The 1/255 that scales states to [0, 1] is applied once
// per output element in the epilogue of the two kernels that read bytes.
static __device__ __forceinline__ void unpack_u8(float (&r)[4], uint32_t w)
{
    r[0] = (float)(w & 255u);
    r[1] = (float)((w >> 8) & 255u);
    r[2] = (float)((w >> 16) & 255u);
    r[3] = (float)(w >> 24);
}
constexpr float STATE_SCALE = 1.0f / 255.0f;
constexpr unsigned ZPB = ZERO_PAGE * 4;      // bytes of zeros in front of every activation buffer

struct OffCtx { unsigned off; };             // byte offset of the group, fixed over the k-loop

struct ProblemBase {
    typedef float4 ARaw;
    typedef float4 BRaw;
    typedef OffCtx CtxA;
    typedef OffCtx CtxB;
    static constexpr bool SUM_A = false, SUM_B = false, HAS_AUX = false, A_ZERO = false, B_ZERO = false;
    static constexpr bool SUMSQ = false;
    static constexpr bool A_EXACT_BF16 = false;   // true: every A value is an integer 0..255 (a byte image)
    static constexpr int PREFETCH = 1;            // k-tiles of global loads in flight (1 or 2)
    static constexpr bool FENCE_STAGING = false;  // bf16 modes: all MFMAs of a tile before the staging of the next
    static constexpr bool PIPELINE = false;       // modes 2, 3: branch-free steady state, two tiles of loads in flight
    static constexpr bool PIPELINE_SINGLE = false; // the same for mode 1
    static constexpr int WAVES_SPLIT3 = 2;         // mode 3: wavefronts per SIMD that the registers must allow
    static constexpr int WAVES = 4;                // the other modes
    static constexpr bool SPLIT3 = false;         // true: fp32 accuracy from three bf16 pieces of both operands
    static constexpr bool A_DIRECT = false;       // true: bf16 modes take A from global memory into the MFMA lanes
    static constexpr bool B_DIRECT = false;       // the same for B
    static constexpr bool DIRECT_SINGLE_PIECE = false;   // whether the bf16 variant (mode 1) does so too
    static constexpr int TABLE = 0;
    static constexpr bool BLOCK_FETCH_A = false;
    __device__ void fill_table(int *, int) {}
    static constexpr bool MFMA16 = GALA_MFMA16;
    int tiles_m, tiles_n, splits;
    int k0, k1;
    __device__ int k_begin() const { return k0; }
    __device__ int k_end() const { return k1; }
    __device__ void bind_tile(int, int) {}
    __device__ int n_ktiles(int bk) const { return (k1 - k0 + bk - 1) / bk; }
    __device__ int ktile_k0(int i, int bk) const { return k0 + i * bk; }
    __device__ void decode_a(float (&r)[4], float4 v, bool) const { unpack(r, v); }
    __device__ void decode_b(float (&r)[4], float4 v, bool) const { unpack(r, v); }
    __device__ float4 col_value4(int) const { return make_float4(0.f, 0.f, 0.f, 0.f); }
    template <bool CHECK> __device__ float4 aux4(int, int) const { return make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ void store_sum_a(int, float) const {}
    __device__ void store_sum_b(int, float) const {}
    template <bool CHECK> __device__ float sumsq4(int, int, float4) const { return 0.f; }
    __device__ void store_sumsq(int, float) const {}
};

// ---- conv1 forward: bytes -> a1 ------------------------------------------------------
// m = (f, oy, ox), n = o, k = (c, kh, kw).  A tile of 16 consecutive k is one channel, two
// kernel rows of eight bytes: the tile-dependent part of the address is uniform.
struct Conv1Fwd : ProblemBase {
    static constexpr int BM = 256, BN = 32, BK = 16, WM = 4, WN = 1;
    static constexpr bool A_KC = true, B_KC = false;
    static constexpr bool A_EXACT_BF16 = true;
    static constexpr int PREFETCH = 2;            // little work per k-tile (byte loads, K = 256): 3 % faster; slower elsewhere
    static constexpr bool PIPELINE = true, PIPELINE_SINGLE = true;      // 110 -> 103 us; bf16 variant 83 -> 81 us
    static constexpr bool FENCE_STAGING = true;   // 4 % faster
    static constexpr bool A_DIRECT = true;        // fp32: 121 -> 116 us; the bf16 variant: 104 -> 83 us
    static constexpr bool DIRECT_SINGLE_PIECE = true;
    typedef uint32_t ARaw;
    struct CtxA { const uint8_t *ptr; };
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
    __device__ void prep_a(CtxA &c, int m, int kl) const
    {
        const int f = m / P1, p = m % P1, oy = p / W1, ox = p % W1;
        const bool roll = f < M;
        const uint8_t *fr = roll ? o_ + (long)f * FRAME : bo_ + (long)(f - M) * FRAME;
        c.ptr = m < rows_ ? fr + (oy * S1 + (kl >> 3)) * W0 + ox * S1 + (kl & 7) : o_;
    }
    __device__ uint32_t fetch_a(CtxA &c, int kt0, bool &) const
    {
        const int koff = (kt0 >> 6) * (H0 * W0) + ((kt0 >> 3) & 7) * W0;      // uniform
        return *reinterpret_cast<const uint32_t *>(c.ptr + koff);
    }
    __device__ void decode_a(float (&r)[4], uint32_t w, bool) const { unpack_u8(r, w); }
    __device__ void prep_b(CtxB &c, int kl, int n) const { c.off = (kl * C1 + n) * 4; }
    __device__ float4 fetch_b(CtxB &c, int kt0, bool &) const { return ldg4b(w_ + kt0 * C1, c.off); }
    __device__ float4 col_value4(int n) const { return *reinterpret_cast<const float4 *>(b_ + n); }
    __device__ bool tile_full(int m0, int) const { return m0 + BM <= rows_; }
    template <bool CHECK> __device__ void store4(int m, int n, float4 v, float4 bias, float4) const
    {
        if (!CHECK || m < rows_) st4(out_ + (long)m * C1 + n, relu_bias4(scale4(v, STATE_SCALE), bias));
    }
};

// ---- conv2 / conv3 forward ---------------------------------------------------------------
// m = (f, oy, ox), n = o, k = (kh, kw, c) over a channels-last input: a tile of 16 consecutive
// k never crosses a kernel row, so its offset is uniform.
template <int CI, int HI, int WI, int CO, int HO, int WO, int KS, int ST>
struct ConvFwd : ProblemBase {
    // One column of wavefronts (32 x 64 each): no two of them read the same input rows, so the input
    // operand skips LDS in mode 3 (conv2 126 -> 120 us, conv3 93 -> 87 us; the bf16 variant is faster
    // through LDS and keeps it).
    static constexpr int BM = 128, BN = 64, BK = 16, WM = 4, WN = 1;
    static constexpr bool A_KC = true, B_KC = false;
    static constexpr bool SPLIT3 = true;
    static constexpr bool A_DIRECT = true;
    static constexpr bool PIPELINE = true, PIPELINE_SINGLE = true;      // conv3: 81 -> 74 us, conv2: 106 -> 104 us; bf16 variant 88 -> 85 us (conv2)
    static_assert((KS * CI) % BK == 0, "a k-tile stays inside one kernel row");
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
    __device__ void prep_a(CtxA &c, int m, int kl) const
    {
        const int f = m / (HO * WO), p = m % (HO * WO), oy = p / WO, ox = p % WO;
        c.off = m < rows_ ? (unsigned)((((f * HI + oy * ST) * WI + ox * ST) * CI + kl) * 4) : 0u;
    }
    __device__ float4 fetch_a(CtxA &c, int kt0, bool &) const
    {
        const int kh = kt0 / (KS * CI), rem = kt0 % (KS * CI);
        return ldg4b(in_ + kh * (WI * CI) + rem, c.off);
    }
    __device__ void prep_b(CtxB &c, int kl, int n) const { c.off = (kl * CO + n) * 4; }
    __device__ float4 fetch_b(CtxB &c, int kt0, bool &) const { return ldg4b(w_ + kt0 * CO, c.off); }
    // Order of the k-tiles: an input element is read by (KS / ST)^2 output positions of a workgroup's rows,
    // through the taps of one parity class (kh % ST, kw % ST).  Per 128-byte line of a pixel's channels the
    // taps of a class are walked back to back (the two 16-channel halves of the line innermost), which
    // brings the reads of the same cache lines within a few k-tiles of each other; in (kh, kw, c) order
    // they lie up to half the loop apart, by which time the lines have left the cache.
    __device__ int ktile_k0(int i, int) const
    {
        static_assert(KS % ST == 0 && CI % 32 == 0 && BK == 16, "parity classes of equal size, whole lines");
        constexpr int Q = KS / ST, TPC = Q * Q, LINES = CI / 32;
        const int half = i % 2, ab = (i / 2) % TPC, cls = (i / (2 * TPC)) % (ST * ST), line = i / (2 * TPC * ST * ST);
        (void)LINES;
        const int kh = cls / ST + ST * (ab / Q), kw = cls % ST + ST * (ab % Q);
        return (kh * KS + kw) * CI + line * 32 + half * BK;
    }
    __device__ float4 col_value4(int n) const { return *reinterpret_cast<const float4 *>(b_ + n); }
    __device__ bool tile_full(int m0, int) const { return m0 + BM <= rows_; }
    template <bool CHECK> __device__ void store4(int m, int n, float4 v, float4 bias, float4) const
    {
        if (!CHECK || m < rows_) st4(out_ + (long)m * CO + n, relu_bias4(v, bias));
    }
};
using Conv2Fwd = ConvFwd<C1, H1, W1, C2, H2, W2, K2, S2>;
using Conv3Fwd = ConvFwd<C2, H2, W2, C3, H3, W3, K3, S3>;

// ---- hidden layer forward (split over k; partial sums to the workspace) -------------------
// m = f, n = j, k = flattened a3.  The row tile is chosen by the number of frames: 96 for a
// learner step (T*B + B frames), 16 or 32 for an acting step (B frames), where the layer is
// bound by streaming its weights and a tall tile would be mostly padding.
template <int BM_>
struct FcFwdT : ProblemBase {
    static constexpr int BM = BM_, BN = 128, BK = 16, WM = 1, WN = 4;
    static constexpr bool PIPELINE_SINGLE = true;  // bf16 variant: 74 -> 69 us; with three pieces the second register set costs a wavefront per SIMD
    static constexpr bool A_KC = true, B_KC = true;
    static constexpr bool SPLIT3 = true;
    static constexpr bool B_DIRECT = true;        // each wavefront has its own 32 weight columns: 82 -> 77 us
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
    __device__ void prep_a(CtxA &c, int m, int kl) const { c.off = m < F ? (unsigned)((m * FLAT + kl) * 4) : 0u; }
    __device__ float4 fetch_a(CtxA &c, int kt0, bool &) const { return ldg4b(a_ + kt0, c.off); }
    __device__ void prep_b(CtxB &c, int kl, int n) const { c.off = (unsigned)((n * FLAT + kl) * 4); }
    __device__ float4 fetch_b(CtxB &c, int kt0, bool &) const { return ldg4b(w_ + kt0, c.off); }
    __device__ bool tile_full(int m0, int) const { return m0 + BM <= F; }
    template <bool CHECK> __device__ void store4(int m, int n, float4 v, float4, float4) const
    {
        if (!CHECK || m < F) st4(out_ + (long)m * FC + n, v);
    }
};
using FcFwd = FcFwdT<96>;

// ---- hidden layer: gradient to a3 (masked by its ReLU) ---------------------------------------
// m = f, n = flattened a3 index, k = j.
struct FcDgrad : ProblemBase {
    static constexpr int BM = 80, BN = 128, BK = 16, WM = 1, WN = 4;     // 5 x 16 rows: no padding at M = 80, 160
    static constexpr bool PIPELINE = true;         // 95 -> 92 us (the bf16 variant: 81 -> 84 us, left as it was)
    static constexpr bool A_KC = true, B_KC = false;
    static constexpr bool HAS_AUX = true;
    static constexpr bool SPLIT3 = true;
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
    __device__ void prep_a(CtxA &c, int m, int kl) const { c.off = m < M ? (unsigned)((m * FC + kl) * 4) : 0u; }
    __device__ float4 fetch_a(CtxA &c, int kt0, bool &) const { return ldg4b(a_ + kt0, c.off); }
    __device__ void prep_b(CtxB &c, int kl, int n) const { c.off = n < FLAT ? (unsigned)((kl * FLAT + n) * 4) : 0u; }
    // every weight is read by one workgroup, once (the forward pass left them in the last-level cache; with the
    // hint they do not displace a3 and dz3: 93 -> 79 us)
    __device__ float4 fetch_b(CtxB &c, int kt0, bool &) const { return ldg4b_stream(w_ + (long)kt0 * FLAT, c.off); }
    __device__ bool tile_full(int m0, int n0) const { return m0 + BM <= M && n0 + BN <= FLAT; }
    template <bool CHECK> __device__ float4 aux4(int m, int n) const
    {
        return ldg4b(act_, (!CHECK || (m < M && n < FLAT)) ? (unsigned)((m * FLAT + n) * 4) : 0u);
    }
    template <bool CHECK> __device__ void store4(int m, int n, float4 v, float4, float4 act) const
    {
        if (!CHECK || (m < M && n < FLAT)) st4(out_ + (long)m * FLAT + n, relu_mask4(v, act));
    }
};

// ---- hidden layer: weight gradient (and bias gradient = sum over frames of dzh) -----------------
// m = j, n = flattened a3 index, k = f.  The number of frames need not be a multiple of the
// k-tile: groups beyond it are read from the start of the buffer and zeroed.
struct FcWgrad : ProblemBase {
    static constexpr int BM = 128, BN = 128, BK = 16, WM = 2, WN = 2;
    static constexpr int WAVES_SPLIT3 = 3;        // 168 registers and 48 KB of tiles: three workgroups per CU instead of two, 73 -> 66 us
    static constexpr bool A_KC = false, B_KC = false;
    static constexpr bool SUM_A = true, A_ZERO = true, B_ZERO = true;
    static constexpr bool SPLIT3 = true;
    static constexpr bool SUMSQ = true;      // this tensor is 95 % of the parameters: its share of ||g||^2
    static constexpr int TILES = (FC / BM) * ((FLAT + BN - 1) / BN);
    static_assert(TILES == FC_WGRAD_TILES && TILES <= NORM_PARTS, "one gradient-norm partial per tile");
    struct CtxA { unsigned off; int kl; };
    struct CtxB { unsigned off; int kl; bool col_ok; };
    const float *dzh, *a3;
    float *g, *norm_part;
    long d_pad, w_off, b_off;
    int M, F;
    const float *a_, *b_;
    float *out_, *bias_, *ssq_;
    __device__ void bind(int agent, int)
    {
        a_ = dzh + (long)agent * M * FC;
        b_ = a3 + (long)agent * F * FLAT;
        out_ = g + agent * d_pad + w_off;
        bias_ = g + agent * d_pad + b_off;
        ssq_ = norm_part + agent * NORM_PARTS;
        k0 = 0; k1 = M;
    }
    template <bool CHECK> __device__ float sumsq4(int, int n, float4 v) const
    {
        return (!CHECK || n < FLAT) ? (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w) : 0.f;
    }
    __device__ void store_sumsq(int tile, float v) const { ssq_[tile] = v; }
    __device__ void store_sum_a(int m, float v) const { bias_[m] = v; }
    __device__ void prep_a(CtxA &c, int m, int kl) const { c.off = (unsigned)((kl * FC + m) * 4); c.kl = kl; }
    __device__ float4 fetch_a(CtxA &c, int kt0, bool &ok) const
    {
        ok = kt0 + c.kl < k1;
        return ldg4b(a_, ok ? c.off + (unsigned)(kt0 * FC * 4) : 0u);
    }
    __device__ void prep_b(CtxB &c, int kl, int n) const
    {
        c.off = (unsigned)((kl * FLAT + n) * 4); c.kl = kl; c.col_ok = n < FLAT;
    }
    __device__ float4 fetch_b(CtxB &c, int kt0, bool &ok) const
    {
        ok = kt0 + c.kl < k1;
        return ldg4b(b_, (ok && c.col_ok) ? c.off + (unsigned)(kt0 * FLAT * 4) : 0u);
    }
    __device__ bool tile_full(int, int n0) const { return n0 + BN <= FLAT; }
    template <bool CHECK> __device__ void store4(int m, int n, float4 v, float4, float4) const
    {
        // 6.4 MB per agent that only the optimizer reads, a whole backward pass later: 66 -> 61.5 us, and the
        // hidden layer's weights stay cached for its data gradient
        if (!CHECK || n < FLAT) st4_stream(out_ + (long)m * FLAT + n, v);
    }
};

// Context of a transposed-convolution row: byte offset of the centre tap inside the zero-paged
// gradient buffer and one validity bit per kernel tap.
struct TapCtx { unsigned off; unsigned mask; };

// ---- conv3: gradient to a2 (stride 1: full correlation with the flipped kernel) -----------------
// m = (iy, ix, f), n = c, k = (kh, kw, o); a tile of 16 consecutive k lies inside one tap.
// Rows are ordered position-major so that a workgroup's rows share two or three input positions:
// the taps that fall outside the 7x7 output for all of them (40 % of all taps on average) are
// left out of its k-loop; a tap that is outside for only some rows is read from the zero page
// in front of dz3 for those rows.  (Sorting the positions by their tap sets would leave out
// another 7 %, but the table look-ups it needs in the epilogue cost more than that: measured.)
// Row -> (position, frame) divides by the runtime frame count with a multiply-high by
// mdiv = 2^32 / M + 1, exact for rows below 2^32 / M (M = 1 needs no division).
struct Conv3Dgrad : ProblemBase {
    static constexpr int BM = 128, BN = 64, BK = 16, WM = 4, WN = 1;
    static constexpr bool A_KC = true, B_KC = true;
    static constexpr bool HAS_AUX = true;
    static constexpr bool SPLIT3 = true;
    static constexpr bool A_DIRECT = true;        // 117 -> 98 us (128-, 192-, 256- and 320-row tiles within 3 us)
    static constexpr int TILES_PER_TAP = C3 / BK;
    typedef TapCtx CtxA;
    const float *dz3, *x, *a2;      // dz3 points at the data; ZERO_PAGE zeros precede the allocation's data
    float *dz2;
    long d_pad, w_off;
    int M, F;
    unsigned mdiv;                  // 2^32 / M + 1
    const float *zp_, *w_, *act_;
    float *out_;
    int rows_;
    unsigned abase_, taps_;         // taps_: taps that are inside for at least one row of the tile
    __device__ void bind(int agent, int)
    {
        zp_ = dz3 - ZERO_PAGE;
        abase_ = ZPB + (unsigned)agent * (unsigned)(M * A3SZ) * 4u;
        w_ = x + agent * d_pad + w_off;
        act_ = a2 + (long)agent * F * A2SZ;
        out_ = dz2 + (long)agent * M * A2SZ;
        rows_ = M * P2;
        k0 = 0; k1 = K3 * K3 * C3;
    }
    static __device__ unsigned tap_mask(int pos)
    {
        const int iy = pos / W2, ix = pos % W2;
        unsigned mask = 0;
#pragma unroll
        for (int t = 0; t < K3 * K3; ++t) {
            const int oy = iy - t / K3, ox = ix - t % K3;
            if (oy >= 0 && oy < H3 && ox >= 0 && ox < W3) mask |= 1u << t;
        }
        return mask;
    }
    __device__ void bind_tile(int m0, int)
    {
        const int last = min(m0 + BM, rows_) - 1;
        taps_ = 0;
        for (int pos = m0 / M; pos <= last / M; ++pos) taps_ |= tap_mask(pos);
    }
    __device__ int n_ktiles(int) const { return __popc(taps_) * TILES_PER_TAP; }
    __device__ int ktile_k0(int i, int) const
    {
        unsigned rest = taps_;
        for (int s = i / TILES_PER_TAP; s > 0; --s) rest &= rest - 1;        // drop the lowest set bits
        return (__ffs(rest) - 1) * C3 + (i % TILES_PER_TAP) * BK;
    }
    __device__ void prep_a(CtxA &c, int m, int kl) const
    {
        const int pos = (M == 1 ? m : (int)__umulhi((unsigned)m, mdiv)), f = m - pos * M, iy = pos / W2, ix = pos % W2;
        c.off = abase_ + (unsigned)((((f * H3 + iy) * W3 + ix) * C3 + kl) * 4);
        c.mask = m < rows_ ? tap_mask(pos) : 0u;
    }
    __device__ float4 fetch_a(CtxA &c, int kt0, bool &) const
    {
        const int t = kt0 / C3, o0 = kt0 % C3, kh = t / K3, kw = t % K3;          // uniform
        const int tap = (o0 - (kh * W3 + kw) * C3) * 4;
        return ldg4b(zp_, ((c.mask >> t) & 1u) ? c.off + (unsigned)tap : 0u);
    }
    __device__ void prep_b(CtxB &c, int kl, int n) const { c.off = (unsigned)((n * C3 + kl) * 4); }
    __device__ float4 fetch_b(CtxB &c, int kt0, bool &) const
    {
        const int t = kt0 / C3, o0 = kt0 % C3;
        return ldg4b(w_ + t * (C2 * C3) + o0, c.off);
    }
    __device__ bool tile_full(int m0, int) const { return m0 + BM <= rows_; }
    // row (position, frame) -> element offset of its channel vector in a [frame][position][C2] tensor
    __device__ unsigned row_off(int m) const
    {
        const int pos = (M == 1 ? m : (int)__umulhi((unsigned)m, mdiv)), f = m - pos * M;
        return (unsigned)((f * P2 + pos) * C2);
    }
    template <bool CHECK> __device__ float4 aux4(int m, int n) const
    {
        return ldg4b(act_, (!CHECK || m < rows_) ? (row_off(m < rows_ ? m : 0) + (unsigned)n) * 4u : 0u);
    }
    template <bool CHECK> __device__ void store4(int m, int n, float4 v, float4, float4 act) const
    {
        if (!CHECK || m < rows_) st4(out_ + row_off(m) + n, relu_mask4(v, act));
    }
};

// ---- conv2: gradient to a1 (stride 2) ----------------------------------------------------------
// Input positions fall into four parity classes (iy%2, ix%2); within a class the transposed
// convolution is a stride-1 2x2 correlation over the same window of dz2, only the kernel taps
// differ.  The four classes therefore form the columns of one GEMM that reads the window once:
// m = (f, y', x') with iy = 2y'+py, n = (class, c), k = (a, b, o) with kh = py + 2a, oy = y' - a.
struct Conv2Dgrad : ProblemBase {
    // (a 4 x 1 wavefront grid with the gradient operand taken straight from global memory reads as
    // much LDS per MFMA as the 2 x 2 grid does and was slower: 130 vs 113 us)
    static constexpr int BM = 128, BN = 128, BK = 16, WM = 2, WN = 2;
    static constexpr bool A_KC = true, B_KC = true;
    static constexpr bool HAS_AUX = true;
    static constexpr bool SPLIT3 = true;
    static constexpr bool FENCE_STAGING = true;   // 128 -> 113 us; neutral or slower for the other kernels
    static constexpr int HY = H1 / 2, WX = W1 / 2, PC = HY * WX;   // 10, 10, 100
    static_assert(BN == 4 * C1, "four classes of C1 channels");
    typedef TapCtx CtxA;
    const float *dz2, *x, *a1;
    float *dz1;
    long d_pad, w_off;
    int M, F;
    const float *zp_, *w_, *act_;
    float *out_;
    int rows_;
    unsigned abase_;
    __device__ void bind(int agent, int)
    {
        zp_ = dz2 - ZERO_PAGE;
        abase_ = ZPB + (unsigned)agent * (unsigned)(M * A2SZ) * 4u;
        w_ = x + agent * d_pad + w_off;
        act_ = a1 + (long)agent * F * A1SZ;
        out_ = dz1 + (long)agent * M * A1SZ;
        rows_ = M * PC;
        k0 = 0; k1 = 4 * C2;
    }
    __device__ void prep_a(CtxA &c, int m, int kl) const
    {
        const int f = m / PC, p = m % PC, yy = p / WX, xx = p % WX;
        c.off = abase_ + (unsigned)((((f * H2 + yy) * W2 + xx) * C2 + kl) * 4);
        unsigned mask = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int oy = yy - (t >> 1), ox = xx - (t & 1);
            if (oy >= 0 && oy < H2 && ox >= 0 && ox < W2) mask |= 1u << t;
        }
        c.mask = m < rows_ ? mask : 0u;
    }
    __device__ float4 fetch_a(CtxA &c, int kt0, bool &) const
    {
        const int t = kt0 / C2, o0 = kt0 % C2;                                     // uniform
        const int tap = (o0 - ((t >> 1) * W2 + (t & 1)) * C2) * 4;
        return ldg4b(zp_, ((c.mask >> t) & 1u) ? c.off + (unsigned)tap : 0u);
    }
    __device__ void prep_b(CtxB &c, int kl, int n) const
    {
        const int cls = n / C1, ch = n % C1;                                       // kernel tap (py, px) of the class
        c.off = (unsigned)(((((cls >> 1) * K2 + (cls & 1)) * C1 + ch) * C2 + kl) * 4);
    }
    __device__ float4 fetch_b(CtxB &c, int kt0, bool &) const
    {
        const int t = kt0 / C2, o0 = kt0 % C2;
        return ldg4b(w_ + (2 * (t >> 1) * K2 + 2 * (t & 1)) * (C1 * C2) + o0, c.off);
    }
    __device__ unsigned out_index(int m, int n) const
    {
        const int f = m / PC, p = m % PC, yy = p / WX, xx = p % WX;
        const int cls = n / C1, ch = n % C1;
        return (unsigned)(((f * H1 + 2 * yy + (cls >> 1)) * W1 + 2 * xx + (cls & 1)) * C1 + ch);
    }
    __device__ bool tile_full(int m0, int) const { return m0 + BM <= rows_; }
    template <bool CHECK> __device__ float4 aux4(int m, int n) const
    {
        return ldg4b(act_, (!CHECK || m < rows_) ? out_index(m, n) * 4u : 0u);
    }
    template <bool CHECK> __device__ void store4(int m, int n, float4 v, float4, float4 act) const
    {
        if (!CHECK || m < rows_) st4(out_ + out_index(m, n), relu_mask4(v, act));
    }
};

// Running position of a weight-gradient thread inside the (frame, oy, ox) reduction index: it
// advances by one k-tile per fetch, so no division is needed inside the loop.
struct WalkCtx { unsigned moff; int p; unsigned foff; int k; };

// ---- conv2 / conv3 weight gradient (split over frames) ----------------------------------------------
// m = (kh, kw, c), n = o, k = (f, oy, ox).  Each split writes MT*CO weight partials followed
// by CO bias partials (the bias gradient is the sum over k of the dz operand).  Both operands
// live in zero-paged buffers: groups past the end of the split's k-range read zeros.
template <int CI, int HI, int WI, int CO, int HO, int WO, int KS, int ST, int BM_>
struct ConvWgrad : ProblemBase {
    static constexpr bool SPLIT3 = true;           // (conv3's 64 x 64 tile: 97 us on fp32 MFMAs, 87 us here; a 192 x 64 tile is
                                                   // faster alone, 75 us, but its 480 workgroups cost the round more beside conv3's data gradient)
    static constexpr int BM = BM_, BN = 64, BK = 16, WM = 2, WN = 2;
    static constexpr bool PIPELINE = true;         // conv3: 88 -> 77 us, conv2: 104 -> 98 us (the bf16 variant: 49 -> 51, 56 -> 59 us, left as it was)
    static constexpr bool A_KC = false, B_KC = false;
    static constexpr bool SUM_B = true;
    static constexpr int MT = KS * KS * CI;
    static constexpr int PART = MT * CO + CO;
    static constexpr int HW = HO * WO;
    static_assert(BK <= HW, "one wrap per tile at most");
    static constexpr int TABLE = HW;  // output position -> byte offset of its window's corner in a frame
    typedef WalkCtx CtxA;
    struct CtxB { unsigned off; int k; };
    const float *in, *dz;           // both preceded by ZERO_PAGE zeros
    float *ws;
    int M, F, fps;
    const float *zin_, *zdz_;
    float *out_;
    const int *tab_;
    unsigned abase_, bbase_;
    __device__ void fill_table(int *tab, int tid)
    {
        tab_ = tab;
        for (int p = tid; p < HW; p += 256) tab[p] = (((p / WO) * ST) * WI + (p % WO) * ST) * CI * 4;
    }
    __device__ void bind(int agent, int split)
    {
        zin_ = in - ZERO_PAGE;
        zdz_ = dz - ZERO_PAGE;
        abase_ = ZPB + (unsigned)agent * (unsigned)(F * (HI * WI * CI)) * 4u;
        bbase_ = ZPB + (unsigned)agent * (unsigned)(M * (HW * CO)) * 4u;
        out_ = ws + ((long)agent * splits + split) * PART;
        k0 = split * fps * HW;
        k1 = min(M, (split + 1) * fps) * HW;
    }
    __device__ void prep_a(CtxA &c, int m, int kl) const
    {
        const int kh = m / (KS * CI), rem = m % (KS * CI);
        c.moff = m < MT ? abase_ + (unsigned)((kh * (WI * CI) + rem) * 4) : 0u;
        c.k = k0 + kl;
        c.p = c.k % HW;
        c.foff = (unsigned)(c.k / HW) * (unsigned)(HI * WI * CI * 4);
    }
    __device__ float4 fetch_a(CtxA &c, int, bool &) const
    {
        const unsigned off = c.moff + c.foff + (unsigned)tab_[c.p];
        const float4 v = ldg4b(zin_, (c.k < k1 && c.moff != 0u) ? off : 0u);
        c.k += BK; c.p += BK;
        if (c.p >= HW) { c.p -= HW; c.foff += (unsigned)(HI * WI * CI * 4); }
        return v;
    }
    __device__ void prep_b(CtxB &c, int kl, int n) const
    {
        c.k = k0 + kl;
        c.off = bbase_ + (unsigned)((c.k * CO + n) * 4);
    }
    __device__ float4 fetch_b(CtxB &c, int, bool &) const
    {
        const float4 v = ldg4b(zdz_, c.k < k1 ? c.off : 0u);
        c.k += BK; c.off += (unsigned)(BK * CO * 4);
        return v;
    }
    __device__ bool tile_full(int m0, int) const { return m0 + BM <= MT; }
    template <bool CHECK> __device__ void store4(int m, int n, float4 v, float4, float4) const
    {
        if (!CHECK || m < MT) st4(out_ + (long)m * CO + n, v);
    }
    __device__ void store_sum_b(int n, float v) const { out_[MT * CO + n] = v; }
};
using Conv2Wgrad = ConvWgrad<C1, H1, W1, C2, H2, W2, K2, S2, 128>;
using Conv3Wgrad = ConvWgrad<C2, H2, W2, C3, H3, W3, K3, S3, 64>;

// ---- conv1 weight gradient (split over frames) ---------------------------------------------------
// m = (c, kh, kw), n = o, k = (f, oy, ox); rollout frames only.  The byte operand comes from
// the caller's buffer (no zero page): groups past the k-range are zeroed after the load.
struct Conv1Wgrad : ProblemBase {
    static constexpr int BM = 256, BN = 32, BK = 16, WM = 4, WN = 1;
    static constexpr bool PIPELINE = true, PIPELINE_SINGLE = true;      // 106 -> 104 us; bf16 variant 100 -> 93 us
    static constexpr int WAVES = 3;                // four would spill to scratch memory (110 instead of 104 us)
    static constexpr bool A_KC = false, B_KC = false;
    static constexpr bool SUM_B = true;
    static constexpr bool A_EXACT_BF16 = true;
    static constexpr int PART = KW1 * C1 + C1;
    static constexpr int TABLE = P1;  // output position -> byte offset of its window's corner in a channel plane
    static constexpr bool BLOCK_FETCH_A = true;
    typedef uint32_t ARaw;
    typedef WalkCtx CtxA;
    struct CtxB { unsigned off; int k; };
    const uint8_t *obs;
    const float *dz1;               // preceded by ZERO_PAGE zeros
    float *ws;
    int M, fps;
    const int *tab_;
    const uint8_t *o_;
    const float *zdz_;
    float *out_;
    unsigned bbase_;
    __device__ void bind(int agent, int split)
    {
        o_ = obs + (long)agent * M * FRAME;
        zdz_ = dz1 - ZERO_PAGE;
        bbase_ = ZPB + (unsigned)agent * (unsigned)(M * A1SZ) * 4u;
        out_ = ws + ((long)agent * splits + split) * PART;
        k0 = split * fps * P1;
        k1 = min(M, (split + 1) * fps) * P1;
    }
    __device__ void prep_a(CtxA &c, int m, int kl) const
    {
        c.moff = (unsigned)((m >> 6) * (H0 * W0) + ((m >> 3) & 7) * W0 + (m & 7));
        c.k = k0 + kl;
        c.p = c.k % P1;
        c.foff = (unsigned)(c.k / P1) * (unsigned)FRAME;
    }
    __device__ void fill_table(int *tab, int tid)
    {
        tab_ = tab;
        for (int p = tid; p < P1; p += 256) tab[p] = ((p / W1) * S1) * W0 + (p % W1) * S1;
    }
    __device__ uint32_t fetch_a(CtxA &c, int, bool &ok) const
    {
        ok = c.k < k1;
        const uint32_t v = ldg_u32b(o_, ok ? c.moff + c.foff + (unsigned)tab_[c.p] : 0u);
        c.k += BK; c.p += BK;
        if (c.p >= P1) { c.p -= P1; c.foff += (unsigned)FRAME; }
        return v;
    }
    // Four groups at consecutive k = four consecutive output positions starting at a multiple of
    // four: they never straddle a frame or an output row (P1, W1 and the k-range bounds are multiples
    // of four), and with stride S1 = 4 bytes between positions their four 4-byte groups are sixteen
    // consecutive bytes of one image row: one walk, one table read and one 16-byte load (4-byte
    // aligned) serve all of them.
    __device__ void fetch_a_block(CtxA &c, int, uint32_t (&raw)[4], bool (&ok)[4]) const
    {
        static_assert(P1 % 4 == 0 && W1 % 4 == 0 && BK % 4 == 0 && S1 == 4, "position quads");
        typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
        const bool in = c.k < k1;
        const unsigned off = in ? c.moff + c.foff + (unsigned)tab_[c.p] : 0u;
        const u32x4_a4 v = *reinterpret_cast<const u32x4_a4 *>(o_ + off);
        raw[0] = v.x; raw[1] = v.y; raw[2] = v.z; raw[3] = v.w;
        ok[0] = ok[1] = ok[2] = ok[3] = in;
        c.k += BK; c.p += BK;
        if (c.p >= P1) { c.p -= P1; c.foff += (unsigned)FRAME; }
    }
    __device__ void decode_a(float (&r)[4], uint32_t w, bool ok) const { unpack_u8(r, ok ? w : 0u); }
    __device__ void prep_b(CtxB &c, int kl, int n) const
    {
        c.k = k0 + kl;
        c.off = bbase_ + (unsigned)((c.k * C1 + n) * 4);
    }
    __device__ float4 fetch_b(CtxB &c, int, bool &) const
    {
        const float4 v = ldg4b(zdz_, c.k < k1 ? c.off : 0u);
        c.k += BK; c.off += (unsigned)(BK * C1 * 4);
        return v;
    }
    __device__ bool tile_full(int, int) const { return true; }
    template <bool CHECK> __device__ void store4(int m, int n, float4 v, float4, float4) const
    {
        st4(out_ + (long)m * C1 + n, scale4(v, STATE_SCALE));
    }
    __device__ void store_sum_b(int n, float v) const { out_[KW1 * C1 + n] = v; }
};

// ---- sum of split-K partials of the convolutions' weight gradients (up to three layers per launch) ----------
// A workgroup owns 1024 consecutive floats of one
// layer's gradient (weights, then bias): out[i] = sum_s part[s][i], partials added in index order, and
// leaves the sum of squares of what it wrote in its slot of the agent's row of gradient-norm partials.
struct ReduceSeg {
    const float *part;      // [N][S][len] partial sums
    int S, blocks, ssq_slot;
    long len, out_off;      // floats per agent and partial; offset of the tensor inside an agent's gradient slice
};

__global__ __launch_bounds__(256) void reduce_grads_kernel(ReduceSeg s3, ReduceSeg s2, ReduceSeg s1, float *g, long d_pad,
                                                           float *ssq)
{
    __shared__ float red[4];
    const int agent = blockIdx.y;
    int b = blockIdx.x;
    // the workgroup's layer (uniform): fields picked one by one, so that the arguments stay in scalar registers
    const int which = b < s3.blocks ? 0 : (b < s3.blocks + s2.blocks ? 1 : 2);
    b -= which == 0 ? 0 : (which == 1 ? s3.blocks : s3.blocks + s2.blocks);
    const float *part = which == 0 ? s3.part : (which == 1 ? s2.part : s1.part);
    const int S = which == 0 ? s3.S : (which == 1 ? s2.S : s1.S);
    const long len = which == 0 ? s3.len : (which == 1 ? s2.len : s1.len);
    const long out_off = which == 0 ? s3.out_off : (which == 1 ? s2.out_off : s1.out_off);
    const int slot = which == 0 ? s3.ssq_slot : (which == 1 ? s2.ssq_slot : s1.ssq_slot);
    const long i = ((long)b * 256 + threadIdx.x) * 4;
    float sq = 0.f;
    if (i < len) {
        const float *p = part + (long)agent * S * len + i;
        float4 acc = *reinterpret_cast<const float4 *>(p);
        // eight partials are requested at a time (the last one again where fewer remain) and added in order
        for (int s0 = 1; s0 < S; s0 += 8) {
            float4 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = *reinterpret_cast<const float4 *>(p + (long)min(s0 + u, S - 1) * len);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < S) { acc.x += t[u].x; acc.y += t[u].y; acc.z += t[u].z; acc.w += t[u].w; }
        }
        *reinterpret_cast<float4 *>(g + agent * d_pad + out_off + i) = acc;
        sq = (acc.x * acc.x + acc.y * acc.y) + (acc.z * acc.z + acc.w * acc.w);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sq;
    __syncthreads();
    if (threadIdx.x == 0) ssq[agent * NORM_PARTS + slot + b] = (red[0] + red[1]) + (red[2] + red[3]);
}

// ---- an agent's statistics of the step, one workgroup per agent, every sum in a fixed order ---------------------
//   stats[0..2]  means over the agent's samples of the policy term, the squared value error and the entropy
//                (one wavefront per term, lane l takes samples l, l + 64, ...)
//   stats[3]     ||g||_2 over all parameters: the partials of the hidden layer's tiles and of the three
//                convolutions' reductions, plus the squares of the tensors behind them in the slice
//                (hidden-layer bias, both heads), which are summed here
//   stats[4]     the clip factor min(1, max_norm / (||g|| + 1e-6))   (Table 2: clip global gradient norm)
__global__ __launch_bounds__(256) void step_stats_kernel(const float *__restrict__ g, long d_pad, long tail_begin,
                                                         const float *__restrict__ ssq, int M,
                                                         const float *__restrict__ loss_part, float max_norm, float *stats)
{
    __shared__ float red[4];
    const int agent = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (wave < 3) {
        float t = 0.f;
        for (int m = lane; m < M; m += 64) t += loss_part[((long)agent * M + m) * 3 + wave];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) t += __shfl_xor(t, off, 64);
        if (lane == 0) stats[agent * 5 + wave] = t * (1.0f / (float)M);
    }
    const float4 *pg = reinterpret_cast<const float4 *>(g + agent * d_pad);
    float acc = 0.f;
#pragma unroll 4
    for (long k = tail_begin / 4 + threadIdx.x; k < d_pad / 4; k += 256) {
        const float4 v = pg[k];
        acc += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
    }
    if (threadIdx.x < NORM_USED) acc += ssq[agent * NORM_PARTS + threadIdx.x];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) red[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float ss = 0.f;
        for (int w = 0; w < 4; ++w) ss += red[w];
        const float norm = sqrtf(ss);
        stats[agent * 5 + 3] = norm;
        stats[agent * 5 + 4] = fminf(1.f, max_norm / (norm + 1e-6f));
    }
}

static constexpr int reduce_blocks(long len) { return (int)((len / 4 + 255) / 256); }

// ---- hidden layer epilogue + heads ---------------------------------------------------------------
// One workgroup of 128 threads per (frame, agent): h = relu(sum of the split-K partials + b_fc),
// four columns per thread, then logits = W_pi h + b_pi (rollout frames) and value = w_v h + b_v
// as block-wide dot products.
__global__ __launch_bounds__(128) void fc_reduce_heads_kernel(const float *__restrict__ part, int S,
                                                              const float *__restrict__ x, Layout L, int M, int F,
                                                              float *h, float *logits, float *values)
{
    __shared__ float red[2][65];
    const int f = blockIdx.x, agent = blockIdx.y, t = threadIdx.x;
    const float *xa = x + agent * L.d_pad;
    const long len = (long)F * FC;
    const float *p = part + (long)agent * S * len + (long)f * FC + t * 4;
    float4 acc = *reinterpret_cast<const float4 *>(p);
    // partials are requested four at a time (the last one again where there are fewer) and added in order
    for (int s0 = 1; s0 < S; s0 += 4) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4 *>(p + (long)min(s0 + u, S - 1) * len);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (s0 + u < S) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
    }
    const float4 b = *reinterpret_cast<const float4 *>(xa + L.fcb + t * 4);
    acc.x = fmaxf(acc.x + b.x, 0.f); acc.y = fmaxf(acc.y + b.y, 0.f);
    acc.z = fmaxf(acc.z + b.z, 0.f); acc.w = fmaxf(acc.w + b.w, 0.f);
    *reinterpret_cast<float4 *>(h + ((long)agent * F + f) * FC + t * 4) = acc;

    const int A = L.n_actions;
    const int n_out = f < M ? A + 1 : 1;            // bootstrap states need the value only
    // HEAD_GROUP outputs at a time: their weight rows are requested together and their reductions
    // interleave, so a workgroup waits for memory once per group rather than once per output
    constexpr int HEAD_GROUP = 4;
    for (int o0 = 0; o0 < n_out; o0 += HEAD_GROUP) {
        float d[HEAD_GROUP];
#pragma unroll
        for (int u = 0; u < HEAD_GROUP; ++u) {
            const int oi = min(o0 + u, n_out - 1);
            const float *w = (oi == n_out - 1) ? xa + L.vw : xa + L.piw + (long)oi * FC;
            const float4 wv = *reinterpret_cast<const float4 *>(w + t * 4);
            d[u] = (wv.x * acc.x + wv.y * acc.y) + (wv.z * acc.z + wv.w * acc.w);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1)
#pragma unroll
            for (int u = 0; u < HEAD_GROUP; ++u) d[u] += __shfl_xor(d[u], off, 64);
        if ((t & 63) == 0)
#pragma unroll
            for (int u = 0; u < HEAD_GROUP; ++u)
                if (o0 + u < n_out) red[t >> 6][o0 + u] = d[u];
    }
    __syncthreads();
    if (t < n_out) {
        const float d = red[0][t] + red[1][t];
        if (t == n_out - 1) values[(long)agent * F + f] = d + xa[L.vb];
        else logits[((long)agent * M + f) * A + t] = d + xa[L.pib + t];
    }
}

// Head parameter gradients: row a < A of W_pi (and b_pi[a]); row A = value head.  One thread
// per (row, column j); frames are summed in four interleaved chains, combined in a fixed order.
__global__ __launch_bounds__(256) void heads_wgrad_kernel(const float *__restrict__ h, Layout L, int M, int F,
                                                          const float *__restrict__ dlogits,
                                                          const float *__restrict__ dvalues, float *g)
{
    const int row = blockIdx.x, agent = blockIdx.y;
    const int j = blockIdx.z * 256 + threadIdx.x;
    const int A = L.n_actions;
    const bool is_v = row == A;
    float *ga = g + agent * L.d_pad;
    const float *hv = h + (long)agent * F * FC + j;
    const float *dp = is_v ? dvalues + (long)agent * M : dlogits + (long)agent * M * A + row;
    const int ds = is_v ? 1 : A;
    float acc[4] = {0.f, 0.f, 0.f, 0.f}, sb[4] = {0.f, 0.f, 0.f, 0.f};
    int f = 0;
    for (; f + 4 <= M; f += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float d = dp[(long)(f + u) * ds];
            acc[u] += d * hv[(long)(f + u) * FC];
            sb[u] += d;
        }
    }
    for (; f < M; ++f) {
        const float d = dp[(long)f * ds];
        acc[0] += d * hv[(long)f * FC];
        sb[0] += d;
    }
    const float w = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    if (is_v) ga[L.vw + j] = w; else ga[L.piw + (long)row * FC + j] = w;
    if (j == 0) {
        const float b = (sb[0] + sb[1]) + (sb[2] + sb[3]);
        if (is_v) ga[L.vb] = b; else ga[L.pib + row] = b;
    }
}

// ---- launch plans --------------------------------------------------------------------------------------

static inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

constexpr int FC_KCHUNK = 784;          // 3136 = 4 * 784
constexpr int FC_KCHUNK_SMALL = 224;    // few frames: twice the splits, so that enough workgroups stream the weights
constexpr int FC_SMALL_FRAMES = 32;
constexpr int FPS_CONV1 = 2, FPS_CONV2 = 8, FPS_CONV3 = 16;   // frames per split of the weight gradients (conv1: at least)
// conv1's weight gradient is one tile per agent and split: enough splits to fill the machine, no more (every split
// is a partial the reduction has to read again: 40 splits of two frames at 32 agents x 80 frames cost 12 us of
// reading, 20 splits of four frames 6 us, with the same kernel time)
static inline int conv1_frames_per_split(int N, int M)
{
    long fps = (long)N * M / 640;                        // about 640 workgroups
    return (int)(fps < FPS_CONV1 ? FPS_CONV1 : (fps > 8 ? 8 : fps));
}

size_t workspace_floats(int N, int M, int F)
{
    size_t need = (size_t)N * cdiv(FLAT, FC_KCHUNK) * F * FC;
    auto mx = [&](size_t v) { if (v > need) need = v; };
    mx((size_t)N * cdiv(FLAT, FC_KCHUNK_SMALL) * FC_SMALL_FRAMES * FC);
    // the three convolutions' weight-gradient partials live side by side until one kernel sums them all
    mx((size_t)N * cdiv(M, FPS_CONV1) * Conv1Wgrad::PART + (size_t)N * cdiv(M, FPS_CONV2) * Conv2Wgrad::PART +
       (size_t)N * cdiv(M, FPS_CONV3) * Conv3Wgrad::PART);
    return need + 1024;
}

// Slots of a row of gradient-norm partials: the hidden layer's tiles, then the workgroups of the
// three convolution weight-gradient reductions.
constexpr int SSQ_CONV1 = FC_WGRAD_TILES;
constexpr int SSQ_CONV2 = SSQ_CONV1 + reduce_blocks(Conv1Wgrad::PART);
constexpr int SSQ_CONV3 = SSQ_CONV2 + reduce_blocks(Conv2Wgrad::PART);
static_assert(SSQ_CONV3 + reduce_blocks(Conv3Wgrad::PART) == NORM_USED && NORM_USED <= 256, "gradient-norm partial slots");

#define GALA_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return e_; } while (0)

hipError_t launch_forward(const NetArgs &a, hipStream_t s, PhaseTimer *pt, hipEvent_t before_fc)
{
    const Layout &L = a.L;
    {
        Conv1Fwd p{};
        p.obs = a.obs; p.boot = a.boot; p.x = a.x; p.a1 = a.b.a1; p.d_pad = L.d_pad; p.w_off = L.w1; p.b_off = L.b1;
        p.M = a.M; p.F = a.F; p.Bn = a.Bn;
        p.tiles_m = cdiv((long)a.F * P1, Conv1Fwd::BM); p.tiles_n = 1; p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s, a.bf16));
        pt->mark("conv1_fwd");
    }
    {
        Conv2Fwd p{};
        p.in = a.b.a1; p.x = a.x; p.out = a.b.a2; p.d_pad = L.d_pad; p.w_off = L.w2; p.b_off = L.b2; p.F = a.F;
        p.tiles_m = cdiv((long)a.F * P2, Conv2Fwd::BM); p.tiles_n = 1; p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s, a.bf16));
        pt->mark("conv2_fwd");
    }
    {
        Conv3Fwd p{};
        p.in = a.b.a2; p.x = a.x; p.out = a.b.a3; p.d_pad = L.d_pad; p.w_off = L.w3; p.b_off = L.b3; p.F = a.F;
        p.tiles_m = cdiv((long)a.F * P3, Conv3Fwd::BM); p.tiles_n = 1; p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s, a.bf16));
        pt->mark("conv3_fwd");
    }
    if (before_fc) GALA_TRY(hipStreamWaitEvent(s, before_fc, 0));
    {
        auto run = [&](auto p, int kchunk) -> hipError_t {
            typedef decltype(p) P;
            p.a3 = a.b.a3; p.x = a.x; p.ws = a.b.ws; p.d_pad = L.d_pad; p.w_off = L.fcw; p.F = a.F;
            p.kchunk = kchunk;
            p.tiles_m = cdiv(a.F, P::BM); p.tiles_n = FC / P::BN; p.splits = cdiv(FLAT, kchunk);
            GALA_TRY(igemm_launch(p, a.N, s, a.bf16));
            pt->mark("fc_fwd");
            hipLaunchKernelGGL(fc_reduce_heads_kernel, dim3(a.F, a.N), dim3(128), 0, s, a.b.ws, p.splits, a.x, L,
                               a.M, a.F, a.b.h, a.b.logits, a.b.values);
            pt->mark("fc_reduce_heads");
            return hipGetLastError();
        };
        if (a.F <= 16) GALA_TRY(run(FcFwdT<16>{}, FC_KCHUNK_SMALL));
        else if (a.F <= FC_SMALL_FRAMES) GALA_TRY(run(FcFwdT<32>{}, FC_KCHUNK_SMALL));
        else GALA_TRY(run(FcFwd{}, FC_KCHUNK));
    }
    return hipGetLastError();
}

// The data-gradient chain heads -> fc -> conv3 -> conv2 is sequential; a layer's weight
// gradient needs only that layer's output gradient.  With a side stream the weight-gradient
// kernels run next to the chain, so that the partly filled last round of workgroups of one
// kernel overlaps work of the other; the same kernels run in both modes, results are identical.
hipError_t launch_backward(const NetArgs &a, const HParams &hp, hipStream_t s, PhaseTimer *pt, const SideStream *side)
{
    const Layout &L = a.L;
    // regions of the workspace for the three convolutions' weight-gradient partials
    const int fps1 = conv1_frames_per_split(a.N, a.M);
    const int S3 = cdiv(a.M, FPS_CONV3), S2 = cdiv(a.M, FPS_CONV2), S1 = cdiv(a.M, fps1);
    float *ws3 = a.b.ws, *ws2 = ws3 + (size_t)a.N * S3 * Conv3Wgrad::PART, *ws1 = ws2 + (size_t)a.N * S2 * Conv2Wgrad::PART;
    const bool fork = side && side->stream && !pt->on;     // per-phase timing needs one stream
    hipStream_t w = fork ? side->stream : s;                // where weight gradients go
    int n_ev = 0;
    // everything enqueued on `s` so far is visible to later work on `w`
    auto publish = [&]() -> hipError_t {
        if (!fork) return hipSuccess;
        hipEvent_t e = side->fork[n_ev++];
        GALA_TRY(hipEventRecord(e, s));
        return hipStreamWaitEvent(w, e, 0);
    };
    // dzh came with the loss
    GALA_TRY(publish());
    hipLaunchKernelGGL(heads_wgrad_kernel, dim3(L.n_actions + 1, a.N, FC / 256), dim3(256), 0, w, a.b.h, L, a.M, a.F,
                       a.b.dlogits, a.b.dvalues, a.b.g);
    GALA_TRY(hipGetLastError());
    pt->mark("heads_wgrad");
    {
        FcWgrad p{};
        p.dzh = a.b.dzh; p.a3 = a.b.a3; p.g = a.b.g; p.d_pad = L.d_pad; p.w_off = L.fcw; p.b_off = L.fcb;
        p.norm_part = a.b.norm_part; p.M = a.M; p.F = a.F;
        p.tiles_m = FC / FcWgrad::BM; p.tiles_n = cdiv(FLAT, FcWgrad::BN); p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, w, a.bf16));
        pt->mark("fc_wgrad");
    }
    {
        FcDgrad p{};
        p.dzh = a.b.dzh; p.x = a.x; p.a3 = a.b.a3; p.dz3 = a.b.dz3; p.d_pad = L.d_pad; p.w_off = L.fcw;
        p.M = a.M; p.F = a.F;
        p.tiles_m = cdiv(a.M, FcDgrad::BM); p.tiles_n = cdiv(FLAT, FcDgrad::BN); p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s, a.bf16));
        pt->mark("fc_dgrad");
    }
    GALA_TRY(publish());
    // conv3
    {
        Conv3Wgrad p{};
        p.in = a.b.a2; p.dz = a.b.dz3; p.ws = ws3; p.M = a.M; p.F = a.F; p.fps = FPS_CONV3;
        p.tiles_m = cdiv(KW3, Conv3Wgrad::BM); p.tiles_n = 1; p.splits = S3;
        GALA_TRY(igemm_launch(p, a.N, w, a.bf16));
        pt->mark("conv3_wgrad");
    }
    {
        Conv3Dgrad p{};
        p.dz3 = a.b.dz3; p.x = a.x; p.a2 = a.b.a2; p.dz2 = a.b.dz2; p.d_pad = L.d_pad; p.w_off = L.w3;
        p.M = a.M; p.F = a.F; p.mdiv = (unsigned)((1ull << 32) / (unsigned)a.M + 1ull);
        p.tiles_m = cdiv((long)a.M * P2, Conv3Dgrad::BM); p.tiles_n = 1; p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s, a.bf16));
        pt->mark("conv3_dgrad");
    }
    GALA_TRY(publish());
    // conv2
    {
        Conv2Wgrad p{};
        p.in = a.b.a1; p.dz = a.b.dz2; p.ws = ws2; p.M = a.M; p.F = a.F; p.fps = FPS_CONV2;
        p.tiles_m = cdiv(KW2, Conv2Wgrad::BM); p.tiles_n = 1; p.splits = S2;
        GALA_TRY(igemm_launch(p, a.N, w, a.bf16));
        pt->mark("conv2_wgrad");
        // the partials of conv3 and conv2 in one launch, beside the data-gradient chain
        ReduceSeg none{nullptr, 0, 0, 0, 0, 0};
        ReduceSeg r3{ws3, S3, reduce_blocks(Conv3Wgrad::PART), SSQ_CONV3, Conv3Wgrad::PART, L.w3};
        ReduceSeg r2{ws2, S2, reduce_blocks(Conv2Wgrad::PART), SSQ_CONV2, Conv2Wgrad::PART, L.w2};
        hipLaunchKernelGGL(reduce_grads_kernel, dim3(r3.blocks + r2.blocks, a.N), dim3(256), 0, w, r3, r2, none, a.b.g,
                           L.d_pad, a.b.norm_part);
        GALA_TRY(hipGetLastError());
        pt->mark("conv32_wgrad_reduce");
    }
    {
        Conv2Dgrad p{};
        p.dz2 = a.b.dz2; p.x = a.x; p.a1 = a.b.a1; p.dz1 = a.b.dz1; p.d_pad = L.d_pad; p.w_off = L.w2;
        p.M = a.M; p.F = a.F;
        p.tiles_m = cdiv((long)a.M * Conv2Dgrad::PC, Conv2Dgrad::BM); p.tiles_n = 1; p.splits = 1;
        GALA_TRY(igemm_launch(p, a.N, s, a.bf16));
        pt->mark("conv2_dgrad");
    }
    // conv1 (the input needs no gradient) follows conv2's data gradient on the same stream: nothing runs beside it
    // any more, and the side stream's last kernel ends long before it does, so neither hand-over is waited for
    if (fork) GALA_TRY(hipEventRecord(side->join, w));
    {
        Conv1Wgrad p{};
        p.obs = a.obs; p.dz1 = a.b.dz1; p.ws = ws1; p.M = a.M; p.fps = fps1;
        p.tiles_m = 1; p.tiles_n = 1; p.splits = S1;
        GALA_TRY(igemm_launch(p, a.N, s, a.bf16));
        pt->mark("conv1_wgrad");
    }
    {
        ReduceSeg none{nullptr, 0, 0, 0, 0, 0};
        ReduceSeg r1{ws1, S1, reduce_blocks(Conv1Wgrad::PART), SSQ_CONV1, Conv1Wgrad::PART, L.w1};
        hipLaunchKernelGGL(reduce_grads_kernel, dim3(r1.blocks, a.N), dim3(256), 0, s, none, none, r1, a.b.g, L.d_pad,
                           a.b.norm_part);
        GALA_TRY(hipGetLastError());
        pt->mark("conv1_wgrad_reduce");
        // every weight gradient is out once the side stream is done too: each agent's statistics
        if (fork) GALA_TRY(hipStreamWaitEvent(s, side->join, 0));
        hipLaunchKernelGGL(step_stats_kernel, dim3(a.N), dim3(256), 0, s, a.b.g, L.d_pad, L.fcb, a.b.norm_part, a.M,
                           a.b.loss_part, hp.max_grad_norm, a.b.stats);
        GALA_TRY(hipGetLastError());
        pt->mark("step_stats");
    }
    return hipSuccess;
}

}  // namespace gala
