// Agent-grouped implicit-GEMM on the gfx950 matrix cores: fp32 MFMA in 32x32x2 or 16x16x4
// blocks, bf16 operands with fp32 accumulation, or fp32 accuracy from bf16 MFMAs on exact bf16
// pieces of the operands (see the MODE list above the kernel).
//
// One launch computes, for every agent, C[m][n] = sum_k A[m][k] * B[k][n] where A and
// B are *views* described by a problem functor P (im2col of an activation tensor, a
// weight matrix, a byte image, ...) and C is consumed four columns at a time by
// P::store4.  The kernel never materialises A or B in HBM: 256 threads stage BM x BK and
// BK x BN tiles through LDS (k-major, so a wavefront's MFMA operand read is one
// ds_read_b32 per lane), double-buffered against the global loads of the next k-tile.
// In the bf16 modes an operand that only one wavefront of the workgroup needs can skip LDS
// (A_DIRECT / B_DIRECT below): its lanes load and split exactly the groups they multiply.
// The result tile leaves through LDS as well, so that every global store (and every
// epilogue operand load) is a float4 with consecutive lanes on consecutive addresses.
//
// P provides
//   static constexpr int  BM, BN, BK        tile sizes (BK multiple of 4)
//   static constexpr int  WM, WN            wavefront grid, WM*WN == 4; each wavefront
//                                           owns (BM/WM) x (BN/WN), multiples of the MFMA block
//   static constexpr bool MFMA16            16x16x4 blocks instead of 32x32x2
//   static constexpr bool A_KC, B_KC        true: the operand is read in groups of 4
//                                           consecutive k; false: 4 consecutive m (or n)
//   int tiles_m, tiles_n, splits            filled by the host
//   void bind(int agent, int split)         per-agent pointers and the split's k-range
//   int  k_begin(), k_end()
//   void bind_tile(int m0, int n0)          optional per-tile set-up after bind (uniform)
//   int  n_ktiles(int bk), ktile_k0(i, bk)  the k-tiles this workgroup visits, in order: by default
//                                           every BK-th k from k_begin(); a functor may leave out tiles
//                                           that are zero for all rows of the workgroup's tile
//   typedef ARaw, BRaw                      what one global load of a group returns (float4, or a
//                                           uint32_t of four bytes)
//   typedef CtxA, CtxB                      per-thread, per-group state prepared once before the
//                                           k-loop (row offsets, tap masks, running positions), so
//                                           that the per-tile address work is a few instructions:
//                                           on this hardware ordinary vector instructions and MFMAs
//                                           share one issue port per SIMD, every VALU instruction in
//                                           the loop is paid for in matrix throughput
//   void prep_a(CtxA &, int m, int kl)      group of rows m.. (A_KC: one row, kl = first local k;
//   void prep_b(CtxB &, int kl, int n)      otherwise 4 rows from m, kl = local k)
//   ARaw fetch_a(CtxA &, int k0, bool &ok)  load the group for the tile starting at k0 (uniform);
//   BRaw fetch_b(CtxB &, int k0, bool &ok)  always issues the load, from a clamped or zero-page
//                                           address when the group does not exist; called once per
//                                           tile with k0 ascending by BK, so it may advance the context
//   static constexpr bool A_ZERO, B_ZERO    the staged values must be zeroed where !ok (operands
//                                           whose invalid groups cannot be read from a zero page)
//   void decode_a(float (&r)[4], ARaw, bool ok)   raw -> four floats (applied at staging time, after
//   void decode_b(float (&r)[4], BRaw, bool ok)   the MFMAs of the current tile were issued)
//   float4 col_value4(int n)                per-column epilogue operand (e.g. the bias), columns n..n+3
//   static constexpr bool HAS_AUX
//   template <bool CHECK> float4 aux4(int m, int n)
//                                           optional per-element epilogue operand (e.g. the activation
//                                           whose sign masks a gradient); loaded from a clamped address
//                                           when CHECK and outside
//   template <bool CHECK> void store4(int m, int n, float4 v, float4 colv, float4 aux)
//   bool tile_full(int m0, int n0)          uniform: the whole BM x BN tile lies inside the output;
//                                           such tiles run the epilogue without bounds tests
//   static constexpr bool SUM_A, SUM_B      optional: also produce sum_k A[m][k] (tiles with
//                                           tn == 0) or sum_k B[k][n] (tiles with tm == 0) over
//                                           the k-range, delivered through store_sum_a(m, v) /
//                                           store_sum_b(n, v); needs the operand in "4 consecutive
//                                           m (n)" mode.  Used for bias gradients, which are exactly
//                                           these sums of an operand the weight-gradient GEMM reads.
//   static constexpr int TABLE              optional: this many ints of LDS for the functor, filled by
//                                           fill_table(int *tab, int tid) (all 256 threads, before the
//                                           first fetch; a barrier follows) and read in fetch_a / fetch_b
//   static constexpr bool BLOCK_FETCH_A     optional, used when a thread owns PA consecutive k of one
//                                           quad of rows (bf16 tiles, m-contiguous A): one call
//                                           fetch_a_block(ctx of the first group, k0, raw[PA], ok[PA])
//                                           loads all of the thread's groups, group i at local k + i
//   static constexpr bool A_EXACT_BF16      optional: every A value is exactly representable in bf16 (a byte
//                                           image); an fp32 run then takes mode 2
//   static constexpr bool A_DIRECT          optional, bf16 modes with WN == 1 and a k-contiguous A: A does not go
//                                           through LDS; every lane loads and splits the groups of its own
//                                           MFMA operand position (prep_a is called with that row and k)
//   static constexpr bool B_DIRECT          the same for a k-contiguous B with WM == 1
//   static constexpr bool DIRECT_SINGLE_PIECE   whether mode 1 (one rounded piece per operand) takes the direct
//                                           path as well: it pays where the operand's loads dominate
//   static constexpr bool SPLIT3            optional: an fp32 run takes mode 3 (both operands as three bf16
//                                           pieces) instead of fp32 MFMAs; set where that is measured faster
//   static constexpr bool FENCE_STAGING     bf16 modes: keep the scheduler from moving staging code (and its wait for
//                                           the global loads) in between the MFMAs of a tile; set where measured faster
//   static constexpr int  PREFETCH          k-tiles of global loads in flight ahead of the MFMAs: 1, or 2 with a
//                                           second set of load registers
//   static constexpr bool PIPELINE          modes 2 and 3: the loop's steady state runs without branches, with two
//                                           tiles of loads in flight and (direct operands) two register sets, so
//                                           that the scheduler may place the staging of tile t + 1 among the MFMAs
//                                           of tile t; set where measured faster (it costs registers)
//   static constexpr bool PIPELINE_SINGLE   the same for mode 1
//   static constexpr int  WAVES_SPLIT3      mode 3: wavefronts per SIMD the register allocation must leave room for
//   static constexpr int  WAVES             the same for the other modes
//   static constexpr bool SUMSQ             optional: the workgroup also delivers the sum of
//                                           squares of what it stored, through
//                                           template <bool CHECK> float sumsq4(m, n, v) (the share of
//                                           one float4 group) and store_sumsq(tile, total), tile =
//                                           tm * tiles_n + tn; summed in a fixed order.  Lets a gradient
//                                           producer supply its part of the gradient norm.
//
// Workgroup ids are interleaved over the 8 XCDs by the dispatcher; the decode below
// keeps all tiles of one agent on one XCD so that its weights and activations are
// shared through that XCD's L2.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>

typedef float gala_f32x16 __attribute__((ext_vector_type(16)));
typedef float gala_f32x4 __attribute__((ext_vector_type(4)));

// One MFMA block: 32x32 (k = 2, 16 accumulator registers) or 16x16 (k = 4, 4 registers).
// Lane l supplies A[row = l % MB][k = l / MB] and B[k = l / MB][col = l % MB]; accumulator
// register v of lane l holds row 8 * (v / 4) + 4 * (l / MB) + v % 4 (the 16x16 block has
// v < 4), column l % MB.
template <bool SMALL> struct MfmaBlock;
template <> struct MfmaBlock<false> {
    static constexpr int MB = 32, KS = 2, NV = 16;
    typedef gala_f32x16 Acc;
    static __device__ __forceinline__ Acc mma(float a, float b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int v, int lk) { return 8 * (v / 4) + 4 * lk + (v % 4); }
};
template <> struct MfmaBlock<true> {
    static constexpr int MB = 16, KS = 4, NV = 4;
    typedef gala_f32x4 Acc;
    static __device__ __forceinline__ Acc mma(float a, float b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int v, int lk) { return 4 * lk + v; }
};

typedef __bf16 gala_bf16x2 __attribute__((ext_vector_type(2)));
typedef float gala_f32x2 __attribute__((ext_vector_type(2)));
typedef short gala_s16x4 __attribute__((ext_vector_type(4)));

typedef __bf16 gala_bf16x8 __attribute__((ext_vector_type(8)));
static __device__ __forceinline__ gala_bf16x8 gala_cat(gala_s16x4 lo, gala_s16x4 hi)
{
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(gala_bf16x8, v);
}

// Three 8-byte operand pieces side by side in six registers, and the two overlapping 16-byte windows of them.
typedef int gala_i32x6 __attribute__((ext_vector_type(6)));
typedef int gala_i32x2 __attribute__((ext_vector_type(2)));
static __device__ __forceinline__ gala_i32x6 gala_win(gala_s16x4 p, gala_s16x4 q, gala_s16x4 r)
{
    const gala_i32x2 P = __builtin_bit_cast(gala_i32x2, p), Q = __builtin_bit_cast(gala_i32x2, q), R = __builtin_bit_cast(gala_i32x2, r);
    return gala_i32x6{P.x, P.y, Q.x, Q.y, R.x, R.y};
}
static __device__ __forceinline__ gala_bf16x8 gala_win_lo(gala_i32x6 w)
{
    return __builtin_bit_cast(gala_bf16x8, __builtin_shufflevector(w, w, 0, 1, 2, 3));
}
static __device__ __forceinline__ gala_bf16x8 gala_win_hi(gala_i32x6 w)
{
    return __builtin_bit_cast(gala_bf16x8, __builtin_shufflevector(w, w, 2, 3, 4, 5));
}

// ds_read_b64_tr_b16: every lane gives the LDS address of four consecutive 16-bit values.  Within each
// block of 16 lanes the 16 x 4 values addressed are taken as four rows of 16 (row r = what lanes 4r .. 4r + 3
// address, in lane order) and arrive transposed: lane i receives column i of rows 0..3 as its four values.
static __device__ __forceinline__ gala_s16x4 gala_lds_read_tr(const unsigned short *p)
{
    typedef gala_s16x4 __attribute__((address_space(3))) *lds_ptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
}

// two floats -> two bf16 (round to nearest even) packed in 32 bits
static __device__ __forceinline__ unsigned gala_pack_bf16(float lo, float hi)
{
    gala_f32x2 v = {lo, hi};
    gala_bf16x2 b = __builtin_convertvector(v, gala_bf16x2);
    return *reinterpret_cast<unsigned *>(&b);
}

// Four fp32 values -> NP bf16 pieces each, as packed pairs (values 0,1 in lo[], 2,3 in hi[]):
// piece q is the round-to-nearest bf16 of what pieces 0..q-1 left over; the leftovers are exact,
// and three pieces add up to the value to 24 significant bits.
template <int NP>
static __device__ __forceinline__ void gala_pieces4(const float (&r)[4], unsigned (&lo)[NP], unsigned (&hi)[NP])
{
    float a0 = r[0], a1 = r[1], a2 = r[2], a3 = r[3];
#pragma unroll
    for (int q = 0; q < NP; ++q) {
        lo[q] = gala_pack_bf16(a0, a1);
        hi[q] = gala_pack_bf16(a2, a3);
        if (q + 1 < NP) {
            a0 -= __uint_as_float(lo[q] << 16); a1 -= __uint_as_float(lo[q] & 0xffff0000u);
            a2 -= __uint_as_float(hi[q] << 16); a3 -= __uint_as_float(hi[q] & 0xffff0000u);
        }
    }
}

// MODE 0: fp32 MFMA as described above.
// MODE 1: the same tiling with operands rounded to bf16 when they are staged into LDS (fp32 in
//   HBM, fp32 accumulation): LDS tiles become [row][k] with k contiguous, one lane reads its four
//   consecutive k as 8 bytes, and each 16x16 block takes one v_mfma_f32_16x16x16_bf16 per 16 k.
// MODE 2: for problems whose A operand is exactly representable in bf16 (P::A_EXACT_BF16: byte
//   images, integers 0..255 have eight significant bits).  A is staged as in MODE 1 without any
//   rounding error, B is staged as three bf16 pieces b0 + b1 + b2 that add up to the fp32 value.
//   Every product is exact in fp32 and the accumulation is fp32, so the result is as accurate as
//   the fp32 MFMA path at a fraction of its matrix time.  Per block and 16 k: one 16x16x32
//   instruction that takes the same four k of b2 and b1 (eight k per lane: two piece products
//   at once), then one 16x16x16 instruction for a b0.
// MODE 3: both operands are staged as three bf16 pieces (each the round-to-nearest bf16 of what
//   the previous ones left over; the leftovers are exact).  With a = a0 + a1 + a2 and
//   b = b0 + b1 + b2 the six products a_p b_q with p + q <= 2 carry the product to 2^-24 of
//   |a||b| (what the three left out add up to at most: half a unit of fp32 round-off of the
//   product); each bf16 product is exact in fp32 and
//   the accumulation is fp32.  Three 16x16x32 instructions per block and 16 k, each adding two piece
//   products (a1 b0 + a0 b2, a0 b1 + a2 b0, a1 b1 + a0 b0: with the pieces of an operand kept side by side
//   in the order 1, 0, 2 every instruction's operand is a window of consecutive registers), take 3/8 of the
//   matrix time of the four fp32 MFMAs they replace.
template <class P, int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(MODE == 3 ? P::WAVES_SPLIT3 : P::WAVES))) void igemm_kernel(P p, int n_agents)
{
    constexpr bool BF16 = MODE != 0;
    constexpr int NA = MODE == 3 ? 3 : 1;                       // bf16 pieces of the A operand
    constexpr int NB = (MODE == 2 || MODE == 3) ? 3 : 1;        // bf16 pieces of the B operand
    static_assert(MODE != 2 || P::A_EXACT_BF16, "three-piece mode needs an A operand that bf16 holds exactly");
    constexpr int BM = P::BM, BN = P::BN, BK = P::BK;
    // fp32 LDS tiles are k-major with a row padding of 16 floats: a wavefront's operand read takes
    // sixteen consecutive floats from each of four consecutive k-rows, and with the rows 16 banks
    // apart (tile widths are multiples of 32) the four groups pair up on the 32 banks without
    // meeting (the bank-conflict counter goes from 39 % of the LDS cycles with 4 floats to 1 %).
    constexpr int SA = BM + 16, SB = BN + 16;
    constexpr int WTM = BM / P::WM, WTN = BN / P::WN;   // wavefront tile
    typedef MfmaBlock<P::MFMA16> Blk;
    constexpr int MB = Blk::MB, NV = Blk::NV;
    constexpr int BI = WTM / MB, BJ = WTN / MB;
    static_assert(P::WM * P::WN == 4, "four wavefronts per workgroup");
    static_assert(WTM % MB == 0 && WTN % MB == 0 && BK % Blk::KS == 0, "wavefront tile in MFMA blocks");
    static_assert(BK % 4 == 0 && BM % 4 == 0 && BN % 4 == 0, "vector groups of four");

    // one LDS allocation: [A tiles x2][B tiles x2] during the k-loop, then the output slab
    constexpr int OFFB = 2 * BK * SA;
    constexpr int SC = BN + 4;                  // row stride of the output slab
    constexpr int SLAB = P::WM * MB;            // rows per epilogue pass: one block-row per wavefront row
    // bf16 tiles of a k-contiguous operand are [piece][row][BK]: four neighbouring lanes store one row's four
    // k-quads (8 bytes each), so sixteen lanes store 128 contiguous bytes, and an MFMA operand read is 8 bytes
    // per lane (sixteen consecutive rows at one k-quad); the quads of a row are exchanged by the row's bits
    // 2..3, which puts the sixteen rows of an operand read on sixteen bank pairs.  Row-contiguous operands
    // use the transposed tiles described below.
    constexpr int RA = BK, RB = BK;                                             // row lengths in shorts
    // A_DIRECT: with one column of wavefronts (WN == 1) no two wavefronts need the same A rows, and a
    // k-contiguous A group (one row, four consecutive k) is exactly what an MFMA lane holds: every
    // lane loads the groups of its own operand position, splits them into pieces in registers and
    // feeds them to the MFMAs; only B goes through LDS.
    constexpr bool A_DIRECT = BF16 && P::A_DIRECT && (MODE != 1 || P::DIRECT_SINGLE_PIECE);
    static_assert(!A_DIRECT || (P::A_KC && P::WN == 1 && !P::SUM_A && P::MFMA16), "direct A operands: k-contiguous, one wavefront column");
    constexpr int NA_LDS = A_DIRECT ? 0 : NA;                                    // pieces of A kept in LDS
    // B_DIRECT: the same for B with one row of wavefronts (WM == 1)
    constexpr bool B_DIRECT = BF16 && P::B_DIRECT && (MODE != 1 || P::DIRECT_SINGLE_PIECE);
    static_assert(!B_DIRECT || (P::B_KC && P::WM == 1 && !P::SUM_B && P::MFMA16 && !A_DIRECT), "direct B operands: k-contiguous, one wavefront row");
    constexpr int NB_LDS = B_DIRECT ? 0 : NB;
    // Row-contiguous operands (weight-gradient operands, weights stored [k][n]) keep their memory order in
    // LDS, [piece][k][row]: a thread stores the four rows it loaded at one k as 8 bytes per piece, and the
    // MFMA operand is fetched by the transposing LDS read of gfx950 (ds_read_b64_tr_b16): within each block
    // of 16 lanes, lane i reads rows 4 (i % 4) .. + 3 at k-row i / 4 and receives row i at those four k.
    // LDS serves these reads 32 lanes (256 bytes, 64 banks) at a time, i.e. two such blocks holding eight
    // consecutive k-rows, and stores 16 lanes (128 bytes) at a time.  Tiles of a multiple of 64 rows have no
    // padding; their 16-row blocks (32 bytes, 8 banks) are exchanged instead.  128 or 256 rows (k-rows start
    // on bank 0): the block index is XORed with (k ^ k / 8) % 8, which puts the eight k-rows of a read on the
    // eight bank groups; where a thread owns consecutive k of one quad of rows (a block fetch), the lanes of
    // one store hold k-rows four apart, which that term separates as well.  64 rows (k-rows alternate between
    // the two halves of the banks): XOR with (k ^ k / 4) % 4.  A k-row's 16 storing lanes write whole
    // 128-byte lines whatever the exchange.  32-row tiles keep 16 shorts of padding per k-row instead, which
    // moves consecutive k-rows by 24 banks: eight of them fall on eight different groups.
    constexpr bool A_TR = BF16 && !P::A_KC, B_TR = BF16 && !P::B_KC;
    constexpr int PITCH_A = BM + (BM % 64 ? 16 : 0), PITCH_B = BN + (BN % 64 ? 16 : 0);   // shorts per k-row of a transposed tile
    constexpr int SZA = A_TR ? BK * PITCH_A : BM * RA, SZB = B_TR ? BK * PITCH_B : BN * RB;   // shorts per piece and buffer
    constexpr int LDS_F32 = 2 * BK * (SA + SB), LDS_BF16 = BF16 ? (2 * (NA_LDS * SZA + NB_LDS * SZB) + 1) / 2 : 0;
    constexpr int LDS_LOOP = BF16 ? LDS_BF16 : LDS_F32, LDS_OUT = SLAB * SC;
    constexpr int LDS_SUMS = (P::SUM_A || P::SUM_B) ? 1024 : 0;
    constexpr int LDS_FLOATS = (LDS_LOOP > LDS_OUT ? LDS_LOOP : LDS_OUT) > LDS_SUMS ? (LDS_LOOP > LDS_OUT ? LDS_LOOP : LDS_OUT) : LDS_SUMS;
    __shared__ __attribute__((aligned(16))) float smem[LDS_FLOATS];
    auto As = [&](int buf, int k, int c) -> float & { return smem[(buf * BK + k) * SA + c]; };
    auto Bs = [&](int buf, int k, int c) -> float & { return smem[OFFB + (buf * BK + k) * SB + c]; };
    // bf16 tiles: [buf][row][BK + 4] shorts (the padding keeps 8-byte alignment and spreads banks)
    static_assert(!BF16 || (P::MFMA16 && BK == 16), "bf16 path: 16x16 blocks, four k-quads per tile row");
    constexpr int OFFBH = 2 * NA_LDS * SZA;
    static_assert(!BF16 || (2 * (NA_LDS * SZA + NB_LDS * SZB) * 2 <= LDS_FLOATS * 4), "bf16 tiles fit the allocation");
    static_assert(OFFBH % 4 == 0 && SZA % 4 == 0 && SZB % 4 == 0, "8-byte aligned tiles");
    unsigned short *hs = reinterpret_cast<unsigned short *>(smem);
    // transposed tiles: the 16-row block a row's block is exchanged with at k-row k (see above)
    auto tr_swz = [](int rows, int k) {
        return rows % 128 == 0 ? ((k ^ (k >> 3)) & 7) << 4 : rows % 64 == 0 ? ((k ^ (k >> 2)) & 3) << 4 : 0;
    };
    auto swz = [](int row, int k) { return k ^ (((row >> 2) & 3) << 2); };
    auto Ah = [&](int buf, int piece, int m, int k) -> unsigned short & {
        if constexpr (A_TR) return hs[(buf * NA + piece) * SZA + k * PITCH_A + (m ^ tr_swz(BM, k))];
        else return hs[((buf * NA + piece) * BM + m) * RA + swz(m, k)];
    };
    auto Bh = [&](int buf, int piece, int n, int k) -> unsigned short & {
        if constexpr (B_TR) return hs[OFFBH + (buf * NB_LDS + piece) * SZB + k * PITCH_B + (n ^ tr_swz(BN, k))];
        else return hs[OFFBH + ((buf * NB_LDS + piece) * BN + n) * RB + swz(n, k)];
    };

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
    p.bind_tile(m0, n0);
    __shared__ __attribute__((aligned(16))) int ftab[P::TABLE > 0 ? P::TABLE : 1];
    if (P::TABLE > 0) {
        p.fill_table(ftab, threadIdx.x);
        __syncthreads();
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wmi = wave / P::WN;
    const int wm0 = wmi * WTM, wn0 = (wave % P::WN) * WTN;

    constexpr int GA = BM * BK / 4, GB = BN * BK / 4;       // groups of four per tile
    constexpr int PA = (GA + 255) / 256, PB = (GB + 255) / 256;
    // Global loads run PF k-tiles ahead of the MFMAs, one register set per tile in flight.
    // PIPE: the k-loop's steady state has no branches and two tiles of loads in flight, so that the staging
    // arithmetic of tile t + 1 (whose loads were issued a whole tile earlier) can be scheduled in between the
    // MFMAs of tile t instead of behind a wait for loads just issued; direct operands take two register sets
    // (one being multiplied, one being filled).
    constexpr bool PIPE = BF16 && (MODE == 1 ? P::PIPELINE_SINGLE : P::PIPELINE);
    constexpr int PF = PIPE ? 2 : P::PREFETCH;
    static_assert(PF == 1 || PF == 2, "one or two k-tiles of loads in flight");
    typename P::ARaw ra[PF][PA];
    typename P::BRaw rb[PF][PB];
    typename P::CtxA ca[PA];
    typename P::CtxB cb[PB];
    bool oka[PF][PA], okb[PF][PB];
    static_assert(!A_DIRECT || PA == BI, "direct A operands: one group per MFMA block row of the wavefront");
    constexpr int NR = PIPE ? 2 : 1;
    gala_s16x4 areg[NR][NA][A_DIRECT ? BI : 1];   // A_DIRECT: the pieces of the tile about to be multiplied
    static_assert(!B_DIRECT || PB == BJ, "direct B operands: one group per MFMA block column of the wavefront");
    gala_s16x4 breg[NR][NB][B_DIRECT ? BJ : 1];
    static_assert(!P::SUM_A || (!P::A_KC && 256 % (BM / 4) == 0), "SUM_A needs m-contiguous groups");
    static_assert(!P::SUM_B || (!P::B_KC && 256 % (BN / 4) == 0), "SUM_B needs n-contiguous groups");
    static_assert(!P::SUM_A || (BM / 4) % (256 / BK) == 0 || PA == 1, "SUM_A: one pass unless k is shared");
    static_assert(!P::SUM_B || (BN / 4) % (256 / BK) == 0 || PB == 1, "SUM_B: one pass unless k is shared");
    float sum_a[PA][4], sum_b[PB][4];
#pragma unroll
    for (int i = 0; i < PA; ++i) sum_a[i][0] = sum_a[i][1] = sum_a[i][2] = sum_a[i][3] = 0.f;
#pragma unroll
    for (int i = 0; i < PB; ++i) sum_b[i][0] = sum_b[i][1] = sum_b[i][2] = sum_b[i][3] = 0.f;
    const bool do_sum_a = P::SUM_A && tn == 0, do_sum_b = P::SUM_B && tm == 0;


    // Group g of an operand read "4 consecutive m (n)" -> (local k, quad index).  When a k-row
    // holds at least 256/BK quads, 256/BK consecutive threads share one k and a thread keeps
    // that k for all of its groups, so whatever the functor derives from k (a position walked
    // through frame, row, column) is computed once per thread and tile, not once per group.
    constexpr int TPK = 256 / BK;                   // threads per k-row in that arrangement
    auto map_mc = [&](auto qc, int i, int &kl, int &q) {
        constexpr int Q = decltype(qc)::value;      // quads per k-row
        if (Q % TPK == 0) { kl = tid / TPK; q = tid % TPK + TPK * i; }
        else { const int g = tid + i * 256; kl = g / Q; q = g % Q; }
    };
    typedef std::integral_constant<int, BM / 4> QA;
    typedef std::integral_constant<int, BN / 4> QB;
    // A functor with a block fetch loads PA consecutive k of one quad of rows per thread (one wide load); the
    // thread then owns a 4 x PA block of the tile and stores it as PA 8-byte k-rows per piece.
    constexpr bool KCONS_A = BF16 && !P::A_KC && !P::SUM_A && GA % 256 == 0 && 256 % (BM / 4) == 0 &&
                             (PA == 2 || PA == 4) && P::BLOCK_FETCH_A;
    constexpr int KT_A = KCONS_A ? 256 / (BM / 4) : 1;          // threads that share a quad of rows
    auto map_a = [&](int i, int &kl, int &q) {
        if (KCONS_A) { kl = (tid % KT_A) * PA + i; q = tid / KT_A; }
        else map_mc(QA{}, i, kl, q);
    };

#pragma unroll
    for (int i = 0; i < PA; ++i) {
        const int g = tid + i * 256;
#pragma unroll
        for (int st = 0; st < PF; ++st) oka[st][i] = true;
        if (GA % 256 == 0 || g < GA) {
            if constexpr (A_DIRECT) p.prep_a(ca[i], m0 + wm0 + i * MB + lane % MB, (lane / MB) * 4);
            else if (P::A_KC) p.prep_a(ca[i], m0 + g / (BK / 4), (g % (BK / 4)) * 4);
            else { int kl, q; map_a(i, kl, q); p.prep_a(ca[i], m0 + q * 4, kl); }
        }
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) {
        const int g = tid + i * 256;
#pragma unroll
        for (int st = 0; st < PF; ++st) okb[st][i] = true;
        if (GB % 256 == 0 || g < GB) {
            if constexpr (B_DIRECT) p.prep_b(cb[i], (lane / MB) * 4, n0 + wn0 + i * MB + lane % MB);
            else if (P::B_KC) p.prep_b(cb[i], (g % (BK / 4)) * 4, n0 + g / (BK / 4));
            else { int kl, q; map_mc(QB{}, i, kl, q); p.prep_b(cb[i], kl, n0 + q * 4); }
        }
    }

    auto fetch = [&](auto setc, int k0) {
        constexpr int st = decltype(setc)::value;
        if constexpr (KCONS_A && P::BLOCK_FETCH_A) p.fetch_a_block(ca[0], k0, ra[st], oka[st]);
        else {
#pragma unroll
            for (int i = 0; i < PA; ++i) {
                const int g = tid + i * 256;
                if (GA % 256 == 0 || g < GA) ra[st][i] = p.fetch_a(ca[i], k0, oka[st][i]);
            }
        }
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            const int g = tid + i * 256;
            if (GB % 256 == 0 || g < GB) rb[st][i] = p.fetch_b(cb[i], k0, okb[st][i]);
        }
    };
    auto stage = [&](auto bufc, auto setc) {
        constexpr int buf = decltype(bufc)::value;
        constexpr int st = decltype(setc)::value;
        if constexpr (KCONS_A) {
            float rr[PA][4];
#pragma unroll
            for (int i = 0; i < PA; ++i) {
                p.decode_a(rr[i], ra[st][i], oka[st][i]);
                if (P::A_ZERO) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) rr[i][j] = oka[st][i] ? rr[i][j] : 0.f;
                }
            }
            int kl, q; map_a(0, kl, q);
#pragma unroll
            for (int i = 0; i < PA; ++i) {                   // four rows at k = kl + i: 8 bytes per piece
                unsigned lo[NA], hi[NA];
                gala_pieces4<NA>(rr[i], lo, hi);
#pragma unroll
                for (int pc = 0; pc < NA; ++pc)
                    *reinterpret_cast<uint2 *>(&Ah(buf, pc, q * 4, kl + i)) = make_uint2(lo[pc], hi[pc]);
            }
        }
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const int g = tid + i * 256;
            if (!KCONS_A && (GA % 256 == 0 || g < GA)) {
                float r[4];
                p.decode_a(r, ra[st][i], oka[st][i]);
                if (P::A_ZERO) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) r[j] = oka[st][i] ? r[j] : 0.f;
                }
                if constexpr (A_DIRECT) {
                    unsigned lo[NA], hi[NA];
                    gala_pieces4<NA>(r, lo, hi);
#pragma unroll
                    for (int pc = 0; pc < NA; ++pc) areg[PIPE ? buf : 0][pc][i] = __builtin_bit_cast(gala_s16x4, make_uint2(lo[pc], hi[pc]));
                } else if (BF16 && P::A_KC) {
                    const int row = g / (BK / 4), kq = g % (BK / 4);
                    unsigned lo[NA], hi[NA];
                    gala_pieces4<NA>(r, lo, hi);
#pragma unroll
                    for (int pc = 0; pc < NA; ++pc)
                        *reinterpret_cast<uint2 *>(&Ah(buf, pc, row, kq * 4)) = make_uint2(lo[pc], hi[pc]);
                } else if (BF16 && A_TR) {
                    int k, mq; map_a(i, k, mq);
                    unsigned lo[NA], hi[NA];
                    gala_pieces4<NA>(r, lo, hi);
#pragma unroll
                    for (int pc = 0; pc < NA; ++pc)
                        *reinterpret_cast<uint2 *>(&Ah(buf, pc, mq * 4, k)) = make_uint2(lo[pc], hi[pc]);
                } else if (P::A_KC) {
                    const int row = g / (BK / 4), kq = g % (BK / 4);
#pragma unroll
                    for (int j = 0; j < 4; ++j) As(buf, kq * 4 + j, row) = r[j];
                } else {
                    int k, mq; map_a(i, k, mq);
                    *reinterpret_cast<float4 *>(&As(buf, k, mq * 4)) = make_float4(r[0], r[1], r[2], r[3]);
                }
                if (!P::A_KC && P::SUM_A && do_sum_a) {     // summed here, not at fetch, so the loads stay in flight
#pragma unroll
                    for (int j = 0; j < 4; ++j) sum_a[i][j] += r[j];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            const int g = tid + i * 256;
            if (GB % 256 == 0 || g < GB) {
                float r[4];
                p.decode_b(r, rb[st][i], okb[st][i]);
                if (P::B_ZERO) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) r[j] = okb[st][i] ? r[j] : 0.f;
                }
                if constexpr (B_DIRECT) {
                    unsigned lo[NB], hi[NB];
                    gala_pieces4<NB>(r, lo, hi);
#pragma unroll
                    for (int pc = 0; pc < NB; ++pc) breg[PIPE ? buf : 0][pc][i] = __builtin_bit_cast(gala_s16x4, make_uint2(lo[pc], hi[pc]));
                } else if (BF16 && P::B_KC) {
                    const int col = g / (BK / 4), kq = g % (BK / 4);
                    unsigned lo[NB], hi[NB];
                    gala_pieces4<NB>(r, lo, hi);
#pragma unroll
                    for (int pc = 0; pc < NB; ++pc)
                        *reinterpret_cast<uint2 *>(&Bh(buf, pc, col, kq * 4)) = make_uint2(lo[pc], hi[pc]);
                } else if (BF16 && B_TR) {
                    int k, nq; map_mc(QB{}, i, k, nq);
                    unsigned lo[NB], hi[NB];
                    gala_pieces4<NB>(r, lo, hi);
#pragma unroll
                    for (int pc = 0; pc < NB; ++pc)
                        *reinterpret_cast<uint2 *>(&Bh(buf, pc, nq * 4, k)) = make_uint2(lo[pc], hi[pc]);
                } else if (P::B_KC) {
                    const int col = g / (BK / 4), kq = g % (BK / 4);
#pragma unroll
                    for (int j = 0; j < 4; ++j) Bs(buf, kq * 4 + j, col) = r[j];
                } else {
                    int k, nq; map_mc(QB{}, i, k, nq);
                    *reinterpret_cast<float4 *>(&Bs(buf, k, nq * 4)) = make_float4(r[0], r[1], r[2], r[3]);
                }
                if (!P::B_KC && P::SUM_B && do_sum_b) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) sum_b[i][j] += r[j];
                }
            }
        }
    };

    typename Blk::Acc acc[BI][BJ];
#pragma unroll
    for (int i = 0; i < BI; ++i)
#pragma unroll
        for (int j = 0; j < BJ; ++j)
#pragma unroll
            for (int v = 0; v < NV; ++v) acc[i][j][v] = 0.f;

    const int lr = lane % MB, lk = lane / MB;
    const int nkt = p.n_ktiles(BK);
    if (nkt > 0) {
        fetch(std::integral_constant<int, 0>{}, p.ktile_k0(0, BK));
        if (PF == 2 && nkt > 1) fetch(std::integral_constant<int, PF - 1>{}, p.ktile_k0(1, BK));
        stage(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    }
    __syncthreads();
    // One k-tile: request the next tile, run this tile's MFMAs out of buffer `buf`, stage the
    // next tile into the other buffer.  `buf` is a compile-time constant (the loop below is
    // unrolled by two) so that every LDS address is a per-lane base plus an immediate.
    auto tile_step = [&](auto bufc, auto fullc, int kt) {
        constexpr int buf = decltype(bufc)::value;
        constexpr bool FULL = decltype(fullc)::value;      // steady state: tiles kt + PF and kt + 1 exist
        // tile kt sits in LDS buffer kt % 2 and came through register set kt % PF
        if (FULL || kt + PF < nkt) fetch(std::integral_constant<int, PF == 2 ? buf : 0>{}, p.ktile_k0(kt + PF, BK));
        // keep the global loads of the next tile ahead of this tile's MFMAs: without the fence
        // the scheduler sinks them next to their first use and their latency is exposed
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (BF16) {
#pragma unroll
            for (int kk = 0; kk < BK; kk += 16) {
                gala_s16x4 a[NA][BI], b[NB][BJ];
#pragma unroll
                for (int pc = 0; pc < NA; ++pc)
#pragma unroll
                    for (int i = 0; i < BI; ++i) {
                        if constexpr (A_DIRECT) a[pc][i] = areg[PIPE ? buf : 0][pc][i];
                        else if constexpr (A_TR) a[pc][i] = gala_lds_read_tr(&Ah(buf, pc, wm0 + i * MB + 4 * (lr & 3), kk + lk * 4 + (lr >> 2)));
                        else a[pc][i] = *reinterpret_cast<const gala_s16x4 *>(&Ah(buf, pc, wm0 + i * MB + lr, kk + lk * 4));
                    }
#pragma unroll
                for (int q = 0; q < NB; ++q)
#pragma unroll
                    for (int j = 0; j < BJ; ++j) {
                        if constexpr (B_DIRECT) b[q][j] = breg[PIPE ? buf : 0][q][j];
                        else if constexpr (B_TR) b[q][j] = gala_lds_read_tr(&Bh(buf, q, wn0 + j * MB + 4 * (lr & 3), kk + lk * 4 + (lr >> 2)));
                        else b[q][j] = *reinterpret_cast<const gala_s16x4 *>(&Bh(buf, q, wn0 + j * MB + lr, kk + lk * 4));
                    }
                // Products of pieces a_pc b_q with pc + q <= NB - 1, the small ones first.  The
                // 16x16x32 instruction takes eight k per lane: fed with the same four k of two
                // different pieces it adds two such products at once.
                if constexpr (MODE == 3) {
                    // pieces side by side in the order (1, 0, 2): the pairs (1, 0) and (0, 2) that the three
                    // instructions take are windows of consecutive registers, no copies
                    gala_i32x6 aw[BI], bw[BJ];
#pragma unroll
                    for (int i = 0; i < BI; ++i) aw[i] = gala_win(a[1][i], a[0][i], a[2][i]);
#pragma unroll
                    for (int j = 0; j < BJ; ++j) bw[j] = gala_win(b[1][j], b[0][j], b[2][j]);
#pragma unroll
                    for (int i = 0; i < BI; ++i)
#pragma unroll
                        for (int j = 0; j < BJ; ++j)       // a1 b0 + a0 b2
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gala_win_lo(aw[i]), gala_win_hi(bw[j]), acc[i][j], 0, 0, 0);
#pragma unroll
                    for (int i = 0; i < BI; ++i)
#pragma unroll
                        for (int j = 0; j < BJ; ++j)       // a0 b1 + a2 b0
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gala_win_hi(aw[i]), gala_win_lo(bw[j]), acc[i][j], 0, 0, 0);
#pragma unroll
                    for (int i = 0; i < BI; ++i)
#pragma unroll
                        for (int j = 0; j < BJ; ++j)       // a1 b1 + a0 b0
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gala_win_lo(aw[i]), gala_win_lo(bw[j]), acc[i][j], 0, 0, 0);
                } else if constexpr (MODE == 2) {
                    // a (b0 + b1 + b2): the two small products in one 16x16x32 instruction, then a b0
                    gala_bf16x8 aa[BI], b21[BJ];
#pragma unroll
                    for (int i = 0; i < BI; ++i) aa[i] = gala_cat(a[0][i], a[0][i]);
#pragma unroll
                    for (int j = 0; j < BJ; ++j) b21[j] = gala_cat(b[2][j], b[1][j]);
#pragma unroll
                    for (int i = 0; i < BI; ++i)
#pragma unroll
                        for (int j = 0; j < BJ; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aa[i], b21[j], acc[i][j], 0, 0, 0);
#pragma unroll
                    for (int i = 0; i < BI; ++i)
#pragma unroll
                        for (int j = 0; j < BJ; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[0][i], b[0][j], acc[i][j], 0, 0, 0);
                } else {
#pragma unroll
                    for (int i = 0; i < BI; ++i)
#pragma unroll
                        for (int j = 0; j < BJ; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[0][i], b[0][j], acc[i][j], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < BK; kk += Blk::KS) {
                float a[BI], b[BJ];
#pragma unroll
                for (int i = 0; i < BI; ++i) a[i] = As(buf, kk + lk, wm0 + i * MB + lr);
#pragma unroll
                for (int j = 0; j < BJ; ++j) b[j] = Bs(buf, kk + lk, wn0 + j * MB + lr);
#pragma unroll
                for (int i = 0; i < BI; ++i)
#pragma unroll
                    for (int j = 0; j < BJ; ++j) acc[i][j] = Blk::mma(a[i], b[j], acc[i][j]);
            }
        }
        // optionally all of this tile's MFMAs are issued before the wave waits for the next tile's global
        // loads: otherwise the scheduler mixes the staging code (and its wait) in between them and the
        // matrix instructions still to come sit behind a memory wait
        if constexpr (BF16 && P::FENCE_STAGING) __builtin_amdgcn_sched_barrier(0);
        if (FULL || kt + 1 < nkt) stage(std::integral_constant<int, buf ^ 1>{}, std::integral_constant<int, PF == 2 ? buf ^ 1 : 0>{});
        __syncthreads();
    };
    int kt = 0;
    if constexpr (PIPE) {
        for (; kt + PF + 1 < nkt; kt += 2) {
            tile_step(std::integral_constant<int, 0>{}, std::true_type{}, kt);
            tile_step(std::integral_constant<int, 1>{}, std::true_type{}, kt + 1);
        }
    }
    for (; kt < nkt; kt += 2) {
        tile_step(std::integral_constant<int, 0>{}, std::false_type{}, kt);
        if (kt + 1 < nkt) tile_step(std::integral_constant<int, 1>{}, std::false_type{}, kt + 1);
    }

    // Operand sums: every thread holds partial sums of the four rows (columns) of each of its
    // groups; the threads that share a quad are combined through LDS in a fixed order.
    if (P::SUM_A || P::SUM_B) {
        float *red = smem;
        static_assert(LDS_FLOATS >= 1024, "LDS scratch for operand sums");
        auto reduce_quads = [&](auto qc, int i, const float (&part)[4], auto &&emit) {
            constexpr int Q = decltype(qc)::value;
            // quads of this pass and the threads that hold each of them
            constexpr bool SHARED_K = Q % TPK == 0;
            constexpr int QP = SHARED_K ? TPK : Q;            // distinct quads in one pass
            constexpr int R = 256 / QP;                       // threads per quad
#pragma unroll
            for (int j = 0; j < 4; ++j) red[tid * 4 + j] = part[j];
            __syncthreads();
            if (tid < QP * 4) {
                const int ql = tid / 4, j = tid & 3;          // thread t of a quad group has tid % QP == ql
                float t = 0.f;
                for (int r = 0; r < R; ++r) t += red[(r * QP + ql) * 4 + j];
                const int quad = SHARED_K ? ql + TPK * i : ql;
                if (SHARED_K || i == 0) emit(quad * 4 + j, t);
            }
            __syncthreads();
        };
        if (P::SUM_A && do_sum_a) {
#pragma unroll
            for (int i = 0; i < PA; ++i)
                reduce_quads(QA{}, i, sum_a[i], [&](int m, float v) { p.store_sum_a(m0 + m, v); });
        }
        if (P::SUM_B && do_sum_b) {
#pragma unroll
            for (int i = 0; i < PB; ++i)
                reduce_quads(QB{}, i, sum_b[i], [&](int n, float v) { p.store_sum_b(n0 + n, v); });
        }
    }

    // Epilogue, one block-row of every wavefront per pass: accumulators -> LDS slab
    // [WM * MB rows][BN], then the workgroup walks the slab in float4 groups, consecutive
    // threads on consecutive columns.  The loop above ended with a barrier, so the slab may
    // overwrite the operand tiles.
    constexpr int GQ = BN / 4;                       // float4 groups per row
    constexpr int GS = SLAB * GQ;                    // groups per slab
    constexpr int PS = (GS + 255) / 256;
    static_assert(256 % GQ == 0 || GQ % 256 == 0 || PS == 1, "a thread keeps its column group across passes");
    float ssq = 0.f;
    auto epilogue = [&](auto checked) {
        constexpr bool CHECK = decltype(checked)::value;
#pragma unroll
        for (int i = 0; i < BI; ++i) {
#pragma unroll
            for (int j = 0; j < BJ; ++j)
#pragma unroll
                for (int v = 0; v < NV; ++v)
                    smem[(wmi * MB + Blk::row(v, lk)) * SC + wn0 + j * MB + lr] = acc[i][j][v];
            __syncthreads();
            float4 val[PS], aux[PS], colv[PS];
            int mm[PS], nn[PS];
#pragma unroll
            for (int s = 0; s < PS; ++s) {
                const int g = tid + s * 256;
                const int q = (GS % 256 == 0 || g < GS) ? g / GQ : 0, nq = g % GQ;
                mm[s] = m0 + (q / MB) * WTM + i * MB + (q % MB);
                nn[s] = n0 + nq * 4;
                aux[s] = P::HAS_AUX ? p.template aux4<CHECK>(mm[s], nn[s]) : make_float4(0.f, 0.f, 0.f, 0.f);
                colv[s] = p.col_value4(nn[s]);
                val[s] = *reinterpret_cast<const float4 *>(&smem[q * SC + nq * 4]);
            }
#pragma unroll
            for (int s = 0; s < PS; ++s) {
                const int g = tid + s * 256;
                if (GS % 256 == 0 || g < GS) {
                    p.template store4<CHECK>(mm[s], nn[s], val[s], colv[s], aux[s]);
                    if (P::SUMSQ) ssq += p.template sumsq4<CHECK>(mm[s], nn[s], val[s]);
                }
            }
            if (i + 1 < BI) __syncthreads();
        }
    };
    if (p.tile_full(m0, n0)) epilogue(std::false_type{});
    else epilogue(std::true_type{});
    if (P::SUMSQ) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ssq += __shfl_xor(ssq, off, 64);
        __syncthreads();
        if (lane == 0) smem[wave] = ssq;
        __syncthreads();
        if (tid == 0) p.store_sumsq(tm * p.tiles_n + tn, (smem[0] + smem[1]) + (smem[2] + smem[3]));
    }
}

// bf16 = false asks for fp32 accuracy: the fp32 MFMA path, or the three-piece bf16 path for
// problems whose A operand bf16 holds exactly (same accuracy, less matrix time).
template <class P>
static inline hipError_t igemm_launch(const P &p, int n_agents, hipStream_t stream, bool bf16 = false)
{
    const int agents_pad = (n_agents + 7) / 8 * 8;
    const int grid = agents_pad * p.tiles_m * p.tiles_n * p.splits;
    if (bf16) hipLaunchKernelGGL((igemm_kernel<P, 1>), dim3(grid), dim3(256), 0, stream, p, n_agents);
    else if constexpr (P::A_EXACT_BF16 && P::MFMA16)
        hipLaunchKernelGGL((igemm_kernel<P, 2>), dim3(grid), dim3(256), 0, stream, p, n_agents);
    else if constexpr (P::SPLIT3 && P::MFMA16)
        hipLaunchKernelGGL((igemm_kernel<P, 3>), dim3(grid), dim3(256), 0, stream, p, n_agents);
    else hipLaunchKernelGGL((igemm_kernel<P, 0>), dim3(grid), dim3(256), 0, stream, p, n_agents);
    return hipGetLastError();
}
