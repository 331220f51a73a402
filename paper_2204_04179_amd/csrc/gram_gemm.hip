// The two dense contractions of the GRAM step, with the dense linear stand-in
// for the content encoder:
//   forward  (Algorithm 1 step 1, Eq. 4):  E[j,:]  = X[uniq[j],:] . W
//   wgrad    (Algorithm 1 step 4, Eq. 7/9): dW[i,c] = sum_s X[item_s, i] * G[s, c]
// bf16 inputs run on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//   forward: k_gemm_nt_bf16, C = A . B^T with both operands stored with the
//            contraction index contiguous: A = rows of X gathered through the
//            unique-ID list inside the tile loads (the unique items' features are
//            never copied), B = W^T.  For large batches its epilogue is the gather
//            as well: every representation is stored straight to the positions of
//            its item.  Small batches take k_encode_bf16.
//   wgrad:   k_wgrad_tn_bf16 contracts over the rows of the gradient buffer, which
//            is the slow dimension of both operands in memory, with transposing
//            LDS reads; split-K over blocks, float32 partials added in split order.
//   Operands are addressed through buffer descriptors (32-bit offsets, out-of-range
//   reads return zero); matrices beyond the 4 GiB a descriptor can address take the
//   WIDE variants of both kernels, which form 64-bit addresses per lane.
// The float32 variants are plain FMA code for small problems.
#include "gram_internal.h"

namespace gram {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void;

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// What a contraction kernel does with an output element before storing it (template parameter
// EPI of the kernels below).  `aux` has the row pitch of C.
//   kEpiPlain      C = v                                   (float32)
//   kEpiReluBf16   C = bf16(max(v, 0))                     (C is a bf16 matrix)
//   kEpiMinus      C = v - aux                             (aux float32: stored targets)
//   kEpiGate       C = v where aux > 0, else 0             (aux bf16: kept activations)
// A row flagged `zero` (the padding item) is stored as zeros in every mode.

// The aux value of an element is fetched ahead of the stores (epi_load for a group of elements,
// then epi_store for the group), so that the loads of a group are in flight together.
template <int EPI>
__device__ __forceinline__ float epi_load(const void* __restrict__ aux, int64_t at)
{
    if (EPI == kEpiMinus) return static_cast<const float*>(aux)[at];
    if (EPI == kEpiGate) {
        const uint16_t a = static_cast<const uint16_t*>(aux)[at];
        return ((a & 0x8000u) || !(a & 0x7fffu)) ? 0.f : 1.f;               // positive bf16 only
    }
    return 0.f;
}

template <int EPI>
__device__ __forceinline__ void epi_store(float* __restrict__ C, int64_t at, float v, float a, bool zero)
{
    if (EPI == kEpiReluBf16) {
        reinterpret_cast<uint16_t*>(C)[at] = (zero || !(v > 0.f)) ? (uint16_t)0 : f32_to_bf16_rne(v);
    } else if (EPI == kEpiMinus) {
        C[at] = zero ? 0.f : v - a;
    } else if (EPI == kEpiGate) {
        C[at] = (zero || a == 0.f) ? 0.f : v;
    } else {
        C[at] = zero ? 0.f : v;
    }
}

// ---- small forward kernel: latency first ------------------------------------------
//
// Batches whose unique items give the 256x256 kernel fewer tiles than there are CUs (and any
// d_in that is not a multiple of 32).  Such a launch is bound by the latency of its loads,
// not by arithmetic: a 64x64 tile per block (one 32x32 MFMA tile per wave) puts a block on
// nearly every CU, K advances in slabs of 64, and the loads of three slabs are in flight in
// registers ahead of the one being multiplied.  Two LDS buffers, one barrier per slab.

constexpr int BM = 64, BN = 64, BK = 64, kSmallDepth = 3;
constexpr int LDS_STRIDE = BK + 8;   // bf16 elements per LDS row (144 bytes: 16-byte aligned, staggers banks)

// W[d_in,d] -> Wt[d,d_in] (bf16)
__global__ __launch_bounds__(kBlock) void k_transpose_u16(const uint16_t* __restrict__ W, int rows,
                                                          int cols, uint16_t* __restrict__ Wt)
{
    __shared__ uint16_t tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    for (int y = ty; y < 32; y += 8)
        if (r0 + y < rows && c0 + tx < cols) tile[y][tx] = W[(int64_t)(r0 + y) * cols + c0 + tx];
    __syncthreads();
    for (int y = ty; y < 32; y += 8)
        if (c0 + y < cols && r0 + tx < rows) Wt[(int64_t)(c0 + y) * rows + r0 + tx] = tile[tx][y];
}

__device__ __forceinline__ uint4 and4(uint4 v, uint32_t m) { return make_uint4(v.x & m, v.y & m, v.z & m, v.w & m); }

// BDIRECT: the second operand is W [d_in, d] as the caller holds it (d a multiple of 8), not its
// transpose: a slab of W is parked as 64 rows of k with 64 values of n each, and the MFMA fragments
// (8 consecutive k for one n) come from the transposing LDS read of gfx950 (ds_read_b64_tr_b16;
// see k_wgrad_tn_bf16 for its lane layout).  Saves the separate transpose launch, which matters
// where this kernel is used: batches that are bound by launch latency.
typedef short sv4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) sv4i16 lds_sv4i16;

template <int EPI, bool BDIRECT = false>
__global__ __launch_bounds__(kBlock) void k_encode_bf16(
    const uint16_t* __restrict__ X, const uint16_t* __restrict__ Wt, const int* __restrict__ uniq,
    const int* __restrict__ u_dev, int d_in, int d, int pad_id, float* __restrict__ E,
    const void* __restrict__ aux)
{
    __shared__ __attribute__((aligned(16))) uint16_t sA[2][BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) uint16_t sB[2][BN * LDS_STRIDE];
    const int U = *u_dev;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    if (m0 >= U) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // each thread moves two 16-byte chunks of A and of B per slab: chunk cid = tid + 256 h is
    // bytes [16 (cid % 8), +16) of row cid / 8.  Rows past the end are clamped to a valid row
    // (their products are never stored); chunks past d_in are loaded from the row's start and
    // replaced by zeros.
    const uint16_t* pa0;
    const uint16_t* pa1;
    const uint16_t* pb0;
    const uint16_t* pb1;
    const int kc0 = (tid & 7) * 8, kc1 = kc0;               // 256 is a multiple of 8: same chunk column
    const int lrow0 = tid >> 3, lrow1 = (tid + kBlock) >> 3;
    {
        const int j0 = m0 + lrow0 < U ? m0 + lrow0 : U - 1, j1 = m0 + lrow1 < U ? m0 + lrow1 : U - 1;
        pa0 = X + (int64_t)uniq[j0] * d_in;
        pa1 = X + (int64_t)uniq[j1] * d_in;
        if (BDIRECT) {
            // chunk of 8 values of n at column n0 + kc0 of row k = slab start + lrow; a column past
            // the matrix is fetched from column 0 (its products are never stored)
            pb0 = pb1 = Wt + (n0 + kc0 < d ? n0 + kc0 : 0);
        } else {
            const int c0 = n0 + lrow0 < d ? n0 + lrow0 : d - 1, c1 = n0 + lrow1 < d ? n0 + lrow1 : d - 1;
            pb0 = Wt + (int64_t)c0 * d_in;
            pb1 = Wt + (int64_t)c1 * d_in;
        }
    }
    uint4 a00, a01, b00, b01, a10, a11, b10, b11, a20, a21, b20, b21;     // three register sets
#define GRAM_LOAD_SLAB(S, K0)                                                                       \
    {                                                                                               \
        const int k_ = (K0) + kc0;                                                                  \
        const int ks_ = k_ < d_in ? k_ : 0;                                                         \
        a##S##0 = *reinterpret_cast<const uint4*>(pa0 + ks_);                                       \
        a##S##1 = *reinterpret_cast<const uint4*>(pa1 + ks_);                                       \
        if (BDIRECT) {                                                                              \
            const int r0_ = (K0) + lrow0 < d_in ? (K0) + lrow0 : 0;                                 \
            const int r1_ = (K0) + lrow1 < d_in ? (K0) + lrow1 : 0;                                 \
            b##S##0 = *reinterpret_cast<const uint4*>(pb0 + (int64_t)r0_ * d);                      \
            b##S##1 = *reinterpret_cast<const uint4*>(pb1 + (int64_t)r1_ * d);                      \
        } else {                                                                                    \
            b##S##0 = *reinterpret_cast<const uint4*>(pb0 + ks_);                                   \
            b##S##1 = *reinterpret_cast<const uint4*>(pb1 + ks_);                                   \
        }                                                                                           \
    }
#define GRAM_PARK_SLAB(S, K0, BUF)                                                                  \
    {                                                                                               \
        const uint32_t keep_ = (K0) + kc0 < d_in ? 0xFFFFFFFFu : 0u;                                \
        *reinterpret_cast<uint4*>(&sA[BUF][lrow0 * LDS_STRIDE + kc0]) = and4(a##S##0, keep_);       \
        *reinterpret_cast<uint4*>(&sA[BUF][lrow1 * LDS_STRIDE + kc1]) = and4(a##S##1, keep_);       \
        const uint32_t kb0_ = BDIRECT ? ((K0) + lrow0 < d_in ? 0xFFFFFFFFu : 0u) : keep_;           \
        const uint32_t kb1_ = BDIRECT ? ((K0) + lrow1 < d_in ? 0xFFFFFFFFu : 0u) : keep_;           \
        *reinterpret_cast<uint4*>(&sB[BUF][lrow0 * LDS_STRIDE + kc0]) = and4(b##S##0, kb0_);        \
        *reinterpret_cast<uint4*>(&sB[BUF][lrow1 * LDS_STRIDE + kc1]) = and4(b##S##1, kb1_);        \
    }

    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    const int nslab = (d_in + BK - 1) / BK;
    const int arow = (wm * 32 + (lane & 31)) * LDS_STRIDE + (lane >> 5) * 8;
    // BDIRECT: sB rows are k; group g = lane / 16 of a transposing read covers k rows
    // (g / 2) * 8 + 4 h + j / 4 and columns wn * 32 + (g % 2) * 16 + 4 (j % 4) .. + 3, j = lane % 16
    const int brow = BDIRECT ? (((lane >> 5) * 8 + ((lane & 15) >> 2)) * LDS_STRIDE + wn * 32 +
                                ((lane >> 4) & 1) * 16 + (lane & 3) * 4)
                             : ((wn * 32 + (lane & 31)) * LDS_STRIDE + (lane >> 5) * 8);
    // slab sl lives in register set sl % 3; in iteration sl the set of slab sl + 1 is parked in
    // the other LDS buffer and refilled with slab sl + 4.  Nothing is conditional (slabs past the
    // end park zeros), so the count of loads in flight is known at every wait.
#define GRAM_SMALL_ITER(SNEXT, SL)                                                                  \
    {                                                                                               \
        GRAM_PARK_SLAB(SNEXT, ((SL) + 1) * BK, ((SL) + 1) & 1)                                      \
        GRAM_LOAD_SLAB(SNEXT, ((SL) + 1 + kSmallDepth) * BK)                                        \
        const uint16_t* a_ = &sA[(SL) & 1][arow];                                                   \
        const uint16_t* b_ = &sB[(SL) & 1][brow];                                                   \
        _Pragma("unroll") for (int ks = 0; ks < BK / 16; ++ks) {                                    \
            const bf16x8 fa = *reinterpret_cast<const bf16x8*>(a_ + ks * 16);                       \
            bf16x8 fb;                                                                              \
            if (BDIRECT) {                                                                          \
                const uint16_t* t_ = b_ + ks * 16 * LDS_STRIDE;                                     \
                const sv4i16 lo_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_sv4i16*)t_);        \
                const sv4i16 hi_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_sv4i16*)(t_ + 4 * LDS_STRIDE)); \
                fb = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7)); \
            } else {                                                                                \
                fb = *reinterpret_cast<const bf16x8*>(b_ + ks * 16);                                \
            }                                                                                       \
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc, 0, 0, 0);                    \
        }                                                                                           \
        __syncthreads();                                                                            \
    }
    GRAM_LOAD_SLAB(0, 0)
    GRAM_LOAD_SLAB(1, BK)
    GRAM_LOAD_SLAB(2, 2 * BK)
    GRAM_PARK_SLAB(0, 0, 0)
    GRAM_LOAD_SLAB(0, 3 * BK)
    __syncthreads();
    for (int s0 = 0; s0 < nslab; s0 += kSmallDepth) {
        GRAM_SMALL_ITER(1, s0)
        GRAM_SMALL_ITER(2, s0 + 1)
        GRAM_SMALL_ITER(0, s0 + 2)
    }
#undef GRAM_LOAD_SLAB
#undef GRAM_PARK_SLAB
#undef GRAM_SMALL_ITER

    // accumulator element r of a lane sits at (row, col) = ((r / 4) * 8 + (lane / 32) * 4 + r % 4, lane % 32)
    const int cc = n0 + wn * 32 + (lane & 31);
    // everything the stores need is fetched first (the aux values and the IDs that tell the padding
    // row): fetched inside the store loop, each store would wait for its own load and, with it, for
    // the stores before it
    float av[16];
    int idr[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int j = m0 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        av[r] = (j < U && cc < d) ? epi_load<EPI>(aux, (int64_t)j * d + cc) : 0.f;
        idr[r] = j < U ? uniq[j] : 0;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int j = m0 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (j < U && cc < d) epi_store<EPI>(E, (int64_t)j * d + cc, acc[r], av[r], idr[r] == pad_id);
    }
}

// ---- C[M,N] = A[M,K] . B[N,K]^T, bf16 in, fp32 out ---------------------------------
//
// 256x256 block tile, K in slabs of 32.  LDS rows are 64 bytes (4 chunks of 16); chunk c
// of row r sits at position c ^ ((r >> 2) & 3), which spreads the 16-byte fragment reads of
// 16 consecutive rows over all banks; the swizzle is applied by choosing which global chunk
// each lane fetches.  Block indices are decoded so that the column tiles of one row tile run
// on the same XCD (consecutive block indices are dealt round-robin to the 8 XCDs) and share
// the strip of A through that XCD's L2.
// Row j of A is A[row_ids[j]]; a row whose ID equals pad_id yields zeros.
constexpr int TM = 256, TN = 256, TK = 32;
constexpr int TROWB = TK * 2;                          // bytes per LDS row
constexpr int TSTAGEB = (TM + TN) * TROWB;             // bytes per stage

// Register-staged loads.  Measured on MI355X: a wave that issues direct-to-LDS loads
// stalls at issue for as long as the memory pipe needs to take them (about 130 cycles
// per 1 KiB instruction at 4 waves per CU), so load time and MFMA time add up.
// buffer_load_dwordx4 into registers issues in about 20 cycles and completes in the
// background.  The kernel therefore loads slab s+3 into one of two register sets, parks
// slab s+1 in LDS (2 stages) just before the barrier that publishes it, and interleaves
// the load, LDS-write and fragment-read instructions with the MFMAs of the current slab.
// Operands are addressed through buffer descriptors (base + 32-bit byte offset); a
// matrix A beyond the 4 GiB such a descriptor can address takes the WIDE variant, whose
// lanes keep 64-bit row pointers instead (every address it forms is a valid one: rows
// past the end are clamped and K is a multiple of the slab).
typedef int v4i32 __attribute__((ext_vector_type(4)));
constexpr int RSTAGES = 2;
constexpr size_t RSMEM = (size_t)RSTAGES * TSTAGEB;
// fused-gather epilogue: 64 staged rows of TN floats (+16 bytes against bank conflicts)
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kScatterRowB = TN * 4 + 16;
constexpr int kScatterTileB = 64 * kScatterRowB;
constexpr size_t RSMEM_SC = 2 * (size_t)kScatterTileB;     // two staging buffers (they overlay the dead stages)
constexpr uint32_t kBufferFlags = 0x00027000;   // raw buffer: 32-bit elements, no swizzle

// NW = waves per block: 4 (each 128x128, one wave per SIMD) or 8 (each 128x64, two per SIMD).
//
// SCATTER (forward only): the epilogue is the gather of Section 3.1 as well.  Row j of the
// product is the representation of unique item j; instead of only storing it to C it is stored
// to H[p,:] for every position p of that item (the positions of item j are perm[seg_off[j] ..
// seg_off[j+1]) in the sorted order of the dedup step), so the representations never make a
// round trip through memory.  Items with more than kLightMax positions are written to C once
// and copied to their positions by k_gather_heavy: a few hundred very popular items own half
// of the positions, and unrolling their copies here would stall a whole tile on one row.
struct ScatterArgs {
    const int* seg_off;   // [U + 1]
    const int* perm;      // [m] positions in sorted order
    void* H;              // [m, ldh] float32, or bf16 with h_bf16 (selects the kernel's HB variant)
    int64_t ldh;
    int write_all;        // also store every row to C (the caller asked for E)
    int h_bf16;
};

// HB (with SCATTER): H holds bf16, values are rounded to nearest even as they are stored.
// BDIRECT: B is not the K-contiguous [n, k] matrix but its transpose as the caller holds it,
// W [k, n] (n a multiple of 8, ldb = n): a slab of it is parked as 32 rows of k with 256 values
// of n each (512-byte rows, 16-byte chunk c of row r at position c ^ ((r & 3) << 2)), and the
// MFMA fragments (8 consecutive k for one n) come from the transposing LDS read, exactly as
// in k_wgrad_tn_bf16 below.  Saves the transposed copy of the weights and its launch.
template <bool GATHER, int NW, bool SCATTER, int EPI = kEpiPlain, bool HB = false, bool WIDE = false,
          bool BDIRECT = false>
__global__ __launch_bounds__(NW * 64) void k_gemm_nt_bf16(
    const uint16_t* __restrict__ A, int64_t lda, uint32_t a_bytes, const int* __restrict__ row_ids,
    const int* __restrict__ m_dev, const uint16_t* __restrict__ B, int64_t ldb, uint32_t b_bytes, int n,
    int ktot, int pad_id, int n_tiles, float* __restrict__ C, int64_t ldc, ScatterArgs sc,
    const void* __restrict__ aux)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    __shared__ int s_pad_row;
    const int M = *m_dev;
    // row tiles are dealt to the XCDs; the column tiles of a row tile stay together
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int m0 = ((q / n_tiles) * 8 + xcd) * TM;
    const int n0 = (q % n_tiles) * TN;
    if (m0 >= M) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NT = NW == 4 ? 4 : 2;          // 32-column MFMA tiles per wave
    constexpr int GA = 16 / NW;                  // 16-row groups of A (and of B) a wave loads per slab
    const int wm = NW == 4 ? wave >> 1 : wave >> 2, wn = NW == 4 ? wave & 1 : wave & 3;
    if (tid == 0) s_pad_row = -1;
    __syncthreads();

    const int nslab = (ktot + TK - 1) / TK;
    constexpr int sl_begin = 0;

    // loader: wave w moves row groups g = GA w + t (16 rows each) of A and of B; lane l moves the
    // chunk that belongs at position l & 3 of row 16 g + (l >> 2).  Rows past M / past n are
    // clamped to a valid row: their products are never stored.
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(A), 0, a_bytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(B), 0, b_bytes, kBufferFlags);
    const int lrow = lane >> 2;
    const int lchunk = (lane & 3) ^ ((lane >> 4) & 3);
    uint32_t oa[GA], ob[GA];
    const unsigned char* pa[WIDE ? GA : 1];
#pragma unroll
    for (int t = 0; t < GA; ++t) {
        const int r = (wave * GA + t) * 16 + lrow;
        const int j = m0 + r < M ? m0 + r : M - 1;
        int64_t rowA = j;
        if (GATHER) {
            const int id = row_ids[j];
            if (m0 + r < M && id == pad_id) s_pad_row = r;   // at most one row is the padding item
            rowA = id;
        }
        oa[t] = (uint32_t)((rowA * lda + (int64_t)sl_begin * TK + lchunk * 8) * 2);
        if (WIDE) pa[t] = reinterpret_cast<const unsigned char*>(A) + (rowA * lda + (int64_t)sl_begin * TK + lchunk * 8) * 2;
        if (BDIRECT) {
            // chunk cb of the slab: row cb / 32 of k, position cb % 32 of that row in LDS; columns past
            // n are clamped to the last chunk (their products are never stored)
            const int cb = (wave * GA + t) * 64 + lane;
            const int krow = cb >> 5;
            int ncol = n0 + (((cb & 31) ^ ((krow & 3) << 2)) << 3);
            if (ncol > n - 8) ncol = n - 8;
            ob[t] = (uint32_t)(((int64_t)krow * ldb + ncol) * 2);
        } else {
            const int nn = n0 + r;
            ob[t] = (uint32_t)(((int64_t)(nn < n ? nn : n - 1) * ldb + (int64_t)sl_begin * TK + lchunk * 8) * 2);
        }
    }
    static_assert(!BDIRECT || NW == 8, "the untransposed second operand is wired for 8 waves");
    const uint32_t b_slab_bytes = BDIRECT ? (uint32_t)(TK * ldb * 2) : (uint32_t)(TK * 2);
    unsigned char* park = smem + (wave * GA) * 1024 + lane * 16;

    // (fused gather) position ranges and position lists of the rows this wave will store in the
    // epilogue; fetched here so that their latency hides behind the contraction
    constexpr int RPW = 64 / NW;             // rows per wave and epilogue round
    int seg_o = 0, seg_n = 0;
    int pv[SCATTER ? 4 * RPW : 1];
    if (SCATTER) {
        {
            const int k = lane & (4 * RPW - 1);
            const int lr = (wave / (NW / 2)) * 128 + (k / RPW) * 32 + (wave % (NW / 2)) * RPW + k % RPW;
            if (m0 + lr < M) {
                seg_o = sc.seg_off[m0 + lr];
                seg_n = sc.seg_off[m0 + lr + 1] - seg_o;
            }
        }
#pragma unroll
        for (int k = 0; k < 4 * RPW; ++k) {
            const int cnt = __builtin_amdgcn_readlane(seg_n, k);
            const int o = __builtin_amdgcn_readlane(seg_o, k);
            pv[k] = (cnt <= kLightMax && lane < cnt) ? sc.perm[o + lane] : 0;
        }
    }

    f32x16 acc[4][NT];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int ph0 = (lane >> 5) ^ ((lane >> 2) & 3);
    const int offA = (wm * 128 + (lane & 31)) * TROWB;
    const int offB = (TM + wn * (NT * 32) + (lane & 31)) * TROWB;
    const int c0 = ph0 * 16, c1 = (ph0 ^ 2) * 16;
    bf16x8 fa[2][4], fb[2][NT];
    v4i32 ra[2][GA], rb[2][GA];
    // (BDIRECT) addresses of the transposing reads: group g = lane / 16, j = lane % 16 (see the header
    // comment of k_wgrad_tn_bf16); the wave's columns start at chunk NT 4 wn of the 512-byte row
    int tr_offB[BDIRECT ? NT : 1];
    if (BDIRECT) {
        const int j16 = lane & 15, grp = lane >> 4;
        const int f_row = (grp >> 1) * 8 + (j16 >> 2);               // + 16 ks + 4 h
        const int f_x = ((j16 >> 2) & 3) << 2;
#pragma unroll
        for (int i = 0; i < NT; ++i)
            tr_offB[i] = TM * TROWB + f_row * 512 +
                         (((wn * (NT * 4) + i * 4 + (grp & 1) * 2 + ((j16 & 3) >> 1)) ^ f_x) * 16) + (j16 & 1) * 8;
    }
#define GRAM_FRAGS(FS, STAGE, COFF, KS)                                                             \
    {                                                                                               \
        const unsigned char* sb_ = smem + (STAGE) * TSTAGEB;                                        \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                               \
            fa[FS][i] = *reinterpret_cast<const bf16x8*>(sb_ + offA + i * 32 * TROWB + (COFF));     \
        _Pragma("unroll") for (int i = 0; i < NT; ++i) {                                            \
            if (BDIRECT) {                                                                          \
                const unsigned char* t_ = sb_ + (KS) * 16 * 512 + tr_offB[i];                       \
                const sv4i16 b0_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_sv4i16*)t_);        \
                const sv4i16 b1_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_sv4i16*)(t_ + 4 * 512)); \
                fb[FS][i] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(b0_, b1_, 0, 1, 2, 3, 4, 5, 6, 7)); \
            } else {                                                                                \
                fb[FS][i] = *reinterpret_cast<const bf16x8*>(sb_ + offB + i * 32 * TROWB + (COFF)); \
            }                                                                                       \
        }                                                                                           \
    }
#define GRAM_MMA(FS)                                                                                \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                   \
        _Pragma("unroll") for (int j = 0; j < NT; ++j)                                              \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[FS][i], fb[FS][j], acc[i][j], 0, 0, 0);
    // Slabs past the end are clamped to the last one (their data is never multiplied).
#define GRAM_LOAD(SET, SLAB)                                                                        \
    {                                                                                               \
        const uint32_t k_ = (uint32_t)(((SLAB) < last ? (SLAB) : last) * (TK * 2));                 \
        const uint32_t kb_ = (uint32_t)((SLAB) < last ? (SLAB) : last) * b_slab_bytes;              \
        _Pragma("unroll") for (int t = 0; t < GA; ++t) {                                            \
            if (WIDE) ra[SET][t] = *reinterpret_cast<const v4i32*>(pa[t] + k_);                      \
            else ra[SET][t] = __builtin_amdgcn_raw_buffer_load_b128(rsA, oa[t] + k_, 0, 0);         \
            rb[SET][t] = __builtin_amdgcn_raw_buffer_load_b128(rsB, ob[t] + kb_, 0, 0);             \
        }                                                                                           \
    }
#define GRAM_PARK(SET, STAGE)                                                                       \
    {                                                                                               \
        unsigned char* p_ = park + (STAGE) * TSTAGEB;                                               \
        _Pragma("unroll") for (int t = 0; t < GA; ++t) {                                            \
            *reinterpret_cast<v4i32*>(p_ + t * 1024) = ra[SET][t];                                  \
            *reinterpret_cast<v4i32*>(p_ + TM * TROWB + t * 1024) = rb[SET][t];                     \
        }                                                                                           \
    }
    // first half of a slab: k-step 0 MFMAs with the k-step 1 fragment reads, then the LDS writes
    // of the next slab, one or two LDS instructions between MFMAs (a burst of LDS instructions
    // blocks the wave at issue while the other waves' bursts drain, and the MFMA pipe idles);
    // second half: k-step 1 MFMAs with the global loads of slab +3 and the fragment reads of the
    // next slab's k-step 0
#define GRAM_SCHED_FIRST                                                                            \
    if (NW == 4) _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                                 \
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                          \
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                                          \
    }                                                                                               \
    if (NW == 4) _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                    \
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                          \
        __builtin_amdgcn_sched_group_barrier(0x200, 2, 0);                                          \
    }
    // (for the gathered forward the compiler's own order measured 2 % faster, for the streamed
    // weight gradient the fixed pattern 25 % faster)
#define GRAM_SCHED_SECOND                                                                           \
    if (!GATHER && NW == 4) {                                                                       \
        _Pragma("unroll") for (int g = 0; g < 8; ++g) {                                             \
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                      \
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                      \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                      \
        }                                                                                           \
    }
#define GRAM_ITER(SL, P)                                                                            \
    {                                                                                               \
        GRAM_FRAGS(1, (SL) & 1, c1, 1)                                                              \
        GRAM_MMA(0)                                                                                 \
        GRAM_PARK(P, ((SL) + 1) & 1)                                                                \
        GRAM_SCHED_FIRST                                                                            \
        __syncthreads();                                                                            \
        GRAM_LOAD(P, (SL) + 3)                                                                      \
        GRAM_FRAGS(0, ((SL) + 1) & 1, c0, 0)                                                        \
        GRAM_MMA(1)                                                                                 \
        GRAM_SCHED_SECOND                                                                           \
    }

    if (nslab > 0) {
        const int last = nslab - 1;
        GRAM_LOAD(0, 0)
        GRAM_LOAD(1, 1)
        GRAM_PARK(0, 0)
        GRAM_LOAD(0, 2)
        __syncthreads();
        GRAM_FRAGS(0, 0, c0, 0)
        int sl = 0;
        for (; sl + 1 < last; sl += 2) {
            GRAM_ITER(sl, 1)          // set 1 holds slab sl+1, set 0 holds slab sl+2
            GRAM_ITER(sl + 1, 0)      // set 0 holds slab sl+2, set 1 holds slab sl+3
        }
        if (sl < last) GRAM_ITER(sl, 1)
        GRAM_FRAGS(1, last & 1, c1, 1)
        GRAM_MMA(0)
        GRAM_MMA(1)
    }

    // accumulator element r of a lane sits at (row, col) = ((r / 4) * 8 + (lane / 32) * 4 + r % 4, lane % 32)
    const int pad_row = GATHER ? s_pad_row : -1;
    if (SCATTER) {
        // The stages are dead.  The tile goes through LDS 64 rows at a time (the 32 rows of MFMA
        // row block i of both wave rows), so that a wave can then store whole 1 KiB row pieces,
        // 16 bytes per lane: once to C for a heavy item, once per position for a light one.
        // Wave w stores rows (w / 4) * 128 + i * 32 + (w % 4) * 8 + u of the tile (u < 8) in round
        // i; lane l < 32 fetches the position range of row i = l / 8, u = l % 8, and the position
        // lists themselves (lane t: position t of the row) are fetched for all 32 rows at once,
        // so their latency is paid once.
        const bool col_ok = n0 + lane * 4 < n;
        // The position lists arrived long ago.  Reading them here once makes the compiler wait for
        // them here once; otherwise every row's store loop would begin with a wait for all vector
        // memory operations, i.e. for the stores of the rows before it.
#pragma unroll
        for (int k = 0; k < 4 * RPW; ++k) asm volatile("" : "+v"(pv[k]));
        __syncthreads();
        // two staging buffers: a wave that has stored its rows of round i stages round i + 1
        // while the others still store, and one barrier per round is enough (round i + 2 reuses
        // the buffer of round i only after the barrier of round i + 1)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            unsigned char* stage = smem + (i & 1) * kScatterTileB;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rr = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                const bool zero = wm * 128 + i * 32 + rr == pad_row;
                float* dst = reinterpret_cast<float*>(stage + (wm * 32 + rr) * kScatterRowB) +
                             wn * (NT * 32) + (lane & 31);
#pragma unroll
                for (int jj = 0; jj < NT; ++jj) dst[jj * 32] = zero ? 0.f : acc[i][jj][r];
            }
            __syncthreads();
            const int cr0 = (wave / (NW / 2)) * 32 + (wave % (NW / 2)) * RPW;           // first staged row
            f32x4 v[RPW];
#pragma unroll
            for (int u = 0; u < RPW; ++u)
                v[u] = *reinterpret_cast<const f32x4*>(stage + (cr0 + u) * kScatterRowB + lane * 16);
#pragma unroll
            for (int u = 0; u < RPW; ++u) {
                const int lr = (cr0 >> 5) * 128 + i * 32 + (cr0 & 31) + u;               // row of the tile
                const int cnt = __builtin_amdgcn_readlane(seg_n, i * RPW + u);
                if (cnt == 0) continue;
                if (cnt > kLightMax || sc.write_all) {
                    if (col_ok) *reinterpret_cast<f32x4*>(C + (int64_t)(m0 + lr) * ldc + n0 + lane * 4) = v[u];
                    if (cnt > kLightMax) continue;
                }
                if (HB) {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 h = {pack_bf16x2(v[u].x, v[u].y), pack_bf16x2(v[u].z, v[u].w)};
                    for (int t = 0; t < cnt; ++t) {
                        const int pos = __builtin_amdgcn_readlane(pv[i * RPW + u], t);
                        if (col_ok)
                            __builtin_nontemporal_store(h, reinterpret_cast<u32x2*>(static_cast<uint16_t*>(sc.H) + (int64_t)pos * sc.ldh + n0 + lane * 4));
                    }
                } else {
                    for (int t = 0; t < cnt; ++t) {
                        const int pos = __builtin_amdgcn_readlane(pv[i * RPW + u], t);
                        if (col_ok)
                            __builtin_nontemporal_store(v[u], reinterpret_cast<f32x4*>(static_cast<float*>(sc.H) + (int64_t)pos * sc.ldh + n0 + lane * 4));
                    }
                }
            }
        }
    } else if (m0 + TM <= M && n0 + TN <= n) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float av[16][NT];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = wm * 128 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                const int64_t at = (int64_t)(m0 + lr) * ldc + n0 + wn * (NT * 32) + (lane & 31);
#pragma unroll
                for (int jj = 0; jj < NT; ++jj) av[r][jj] = epi_load<EPI>(aux, at + jj * 32);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = wm * 128 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                const int64_t at = (int64_t)(m0 + lr) * ldc + n0 + wn * (NT * 32) + (lane & 31);
                const bool zero = lr == pad_row;
#pragma unroll
                for (int jj = 0; jj < NT; ++jj) epi_store<EPI>(C, at + jj * 32, acc[i][jj][r], av[r][jj], zero);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float av[16][NT];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = wm * 128 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                const int64_t at = (int64_t)(m0 + lr) * ldc + n0 + wn * (NT * 32) + (lane & 31);
#pragma unroll
                for (int jj = 0; jj < NT; ++jj)
                    av[r][jj] = (m0 + lr < M && n0 + wn * (NT * 32) + jj * 32 + (lane & 31) < n)
                                    ? epi_load<EPI>(aux, at + jj * 32) : 0.f;
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = wm * 128 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                if (m0 + lr < M) {
                    const int64_t at = (int64_t)(m0 + lr) * ldc + n0 + wn * (NT * 32) + (lane & 31);
                    const bool zero = lr == pad_row;
#pragma unroll
                    for (int jj = 0; jj < NT; ++jj)
                        if (n0 + wn * (NT * 32) + jj * 32 + (lane & 31) < n)
                            epi_store<EPI>(C, at + jj * 32, acc[i][jj][r], av[r][jj], zero);
                }
            }
        }
    }
}
#undef GRAM_FRAGS
#undef GRAM_MMA
#undef GRAM_LOAD
#undef GRAM_PARK
#undef GRAM_SCHED_FIRST
#undef GRAM_SCHED_SECOND
#undef GRAM_ITER

constexpr int kGemmWaves = 8;

template <bool SCATTER, int EPI, bool HB, bool WIDE, bool BDIRECT = false>
static void launch_gemm_variant(Ctx* c, int kid, unsigned blocks, hipStream_t s, const uint16_t* A, int64_t lda,
                                int64_t a_bytes, const int* row_ids, const int* m_dev, const uint16_t* B,
                                int64_t ldb, int64_t b_bytes, int n, int k, int pad_id, int n_tiles, float* C,
                                int64_t ldc, const ScatterArgs& sc, const void* aux)
{
    constexpr auto kern = k_gemm_nt_bf16<true, kGemmWaves, SCATTER, EPI, HB, WIDE, BDIRECT>;
    constexpr size_t smem = SCATTER ? RSMEM_SC : RSMEM;
    ensure_dynamic_lds<kern>((int)smem);
    // the descriptor of a WIDE operand is not used; any size that fits its field will do
    launch_smem(c, kid, kern, dim3(blocks), dim3(kGemmWaves * 64), smem, s, A, lda,
                (uint32_t)(WIDE ? 0 : a_bytes), row_ids, m_dev, B, ldb, (uint32_t)b_bytes, n, k, pad_id, n_tiles, C,
                ldc, sc, aux);
}

// C[j,:] = epi(A[row_ids[j],:k] . B^T) for j < *m_dev <= m_bound with the 256x256 kernel.
// a_rows / b_rows: rows of the matrices A and B as allocated (A: all rows that row_ids may
// name).  A may lie beyond 4 GiB for the plain epilogue (with or without the fused gather);
// the other epilogue modes and B need buffer descriptors (callers check).
// b_direct: B is the [k, n] matrix as the caller holds it (ldb = n, b_rows = k, n a multiple of 8)
// instead of its K-contiguous transpose; available for A below 4 GiB and every mode but "gate".
static void launch_gemm_nt(Ctx* c, const uint16_t* A, int64_t lda, int64_t a_rows, const int* row_ids,
                           const int* m_dev, int64_t m_bound, const uint16_t* B, int64_t ldb, int64_t b_rows,
                           int n, int k, float* C, int64_t ldc, hipStream_t s, const ScatterArgs* scatter,
                           int pad_id, int epi, const void* aux, bool b_direct = false)
{
    const int n_tiles = (n + TN - 1) / TN;
    const unsigned blocks = (unsigned)((((m_bound + TM - 1) / TM + 7) / 8 * 8) * n_tiles);
    const int64_t a_bytes = a_rows * lda * 2, b_bytes = b_rows * ldb * 2;
    const bool wide = a_bytes >= kBufferWindow;
    const int kid = wide ? KID_ENCODE_BF16_WIDE : KID_ENCODE_BF16;
    const ScatterArgs none = {nullptr, nullptr, nullptr, 0, 0, 0};
#define GRAM_GO(SC, EPI, HB, WIDE, ARGS)                                                            \
    launch_gemm_variant<SC, EPI, HB, WIDE>(c, kid, blocks, s, A, lda, a_bytes, row_ids, m_dev, B, ldb, b_bytes, n, \
                                           k, pad_id, n_tiles, C, ldc, ARGS, aux)
#define GRAM_GO_DIRECT(SC, EPI, HB, ARGS)                                                           \
    launch_gemm_variant<SC, EPI, HB, false, true>(c, kid, blocks, s, A, lda, a_bytes, row_ids, m_dev, B, ldb, b_bytes, n, \
                                                  k, pad_id, n_tiles, C, ldc, ARGS, aux)
    if (b_direct) {
        if (epi == kEpiReluBf16) GRAM_GO_DIRECT(false, kEpiReluBf16, false, none);
        else if (epi == kEpiMinus) GRAM_GO_DIRECT(false, kEpiMinus, false, none);
        else if (scatter && scatter->h_bf16) GRAM_GO_DIRECT(true, kEpiPlain, true, *scatter);
        else if (scatter) GRAM_GO_DIRECT(true, kEpiPlain, false, *scatter);
        else GRAM_GO_DIRECT(false, kEpiPlain, false, none);
    } else if (epi == kEpiReluBf16) GRAM_GO(false, kEpiReluBf16, false, false, none);
    else if (epi == kEpiMinus) GRAM_GO(false, kEpiMinus, false, false, none);
    else if (epi == kEpiGate) GRAM_GO(false, kEpiGate, false, false, none);
    else if (scatter && scatter->h_bf16) {
        if (wide) GRAM_GO(true, kEpiPlain, true, true, *scatter);
        else GRAM_GO(true, kEpiPlain, true, false, *scatter);
    } else if (scatter) {
        if (wide) GRAM_GO(true, kEpiPlain, false, true, *scatter);
        else GRAM_GO(true, kEpiPlain, false, false, *scatter);
    } else {
        if (wide) GRAM_GO(false, kEpiPlain, false, true, none);
        else GRAM_GO(false, kEpiPlain, false, false, none);
    }
#undef GRAM_GO
#undef GRAM_GO_DIRECT
}

// ---- 64x64 bf16 transpose through LDS (16-byte global accesses both ways) ----------

constexpr int TT = 64;   // transpose tile edge

// Wt[cols, rows] = W[rows, cols]^T; rows and cols multiples of 8.
__global__ __launch_bounds__(kBlock) void k_transpose_w(const uint16_t* __restrict__ W, int rows, int cols,
                                                        uint16_t* __restrict__ Wt)
{
    __shared__ uint16_t tile[TT][TT + 2];     // [row of W][column of W]
    const int r_tiles = (rows + TT - 1) / TT, c_tiles = (cols + TT - 1) / TT;
    for (int t = blockIdx.x; t < r_tiles * c_tiles; t += gridDim.x) {
        const int r0 = (t / c_tiles) * TT, c0 = (t % c_tiles) * TT;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int cid = threadIdx.x + h * kBlock;
            const int row = cid >> 3, ch = (cid & 7) * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (r0 + row < rows && c0 + ch < cols)
                v = *reinterpret_cast<const uint4*>(W + (int64_t)(r0 + row) * cols + c0 + ch);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) tile[row][ch + e] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
        }
        __syncthreads();
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int cid = threadIdx.x + h * kBlock;
            const int r = cid >> 3, ch = (cid & 7) * 8;
            if (c0 + r < cols && r0 + ch < rows) {
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    w[e] = (uint32_t)tile[ch + 2 * e][r] | ((uint32_t)tile[ch + 2 * e + 1][r] << 16);
                *reinterpret_cast<uint4*>(Wt + (int64_t)(c0 + r) * rows + r0 + ch) = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
        __syncthreads();
    }
}

// ---- forward, float32 --------------------------------------------------------

__global__ __launch_bounds__(kBlock) void k_encode_f32(
    const float* __restrict__ X, const float* __restrict__ W, const int* __restrict__ uniq,
    const int* __restrict__ u_dev, int d_in, int d, int pad_id, float* __restrict__ E)
{
    const int U = *u_dev;
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int j = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (j >= U || c >= d) return;
    const int id = uniq[j];
    float acc = 0.f;
    if (id != pad_id) {
        const float* x = X + (int64_t)id * d_in;
        for (int k = 0; k < d_in; ++k) acc = fmaf(x[k], W[(int64_t)k * d + c], acc);
    }
    E[(int64_t)j * d + c] = acc;
}

// Wt[cols, rows] = W[rows, cols]^T for a bf16 matrix whose rows count is a multiple of 8.
void transpose_weight(Ctx* c, const void* W, int rows, int cols, void* Wt, hipStream_t s)
{
    // 16-byte row chunks of W^T never straddle its end because rows is a multiple of 8
    if (cols % 8 == 0) {
        const int tiles = ((rows + TT - 1) / TT) * ((cols + TT - 1) / TT);
        launch(c, KID_TRANSPOSE_U16, k_transpose_w, dim3(tiles < 1024 ? tiles : 1024), dim3(kBlock), s,
               static_cast<const uint16_t*>(W), rows, cols, static_cast<uint16_t*>(Wt));
    } else {
        launch(c, KID_TRANSPOSE_U16, k_transpose_u16, dim3((cols + 31) / 32, (rows + 31) / 32), dim3(kBlock), s,
               static_cast<const uint16_t*>(W), rows, cols, static_cast<uint16_t*>(Wt));
    }
}

// Batches that give the 256x256 kernel a tile for every CU (and a K that fits its slabs) take it;
// the rest take the 64x64 latency-oriented kernel, which addresses its operands through plain
// pointers and therefore also serves the epilogue modes when A lies beyond 4 GiB.
static bool takes_big_kernel(const Ctx* c, int64_t rows_max, int n_out, int k, int64_t a_rows, int epi)
{
    const int64_t tile_bound = ((rows_max + TM - 1) / TM) * ((n_out + TN - 1) / TN);
    if (epi != kEpiPlain && a_rows * k * 2 >= kBufferWindow) return false;
    return tile_bound >= c->num_cus && k % TK == 0;
}

// The 256x256 kernel reads the second operand untransposed for these shapes and modes.
static bool big_kernel_reads_plain_b(int64_t a_rows, int k, int n_out, int epi)
{
    return n_out % 8 == 0 && n_out >= 8 && epi != kEpiGate && a_rows * k * 2 < kBufferWindow &&
           (int64_t)k * n_out * 2 < kBufferWindow;
}

// Whether gemm_rows_bf16 will read B_plain (the [k, n_out] matrix as the caller holds it) instead of
// the transposed copy Bt for this problem: callers skip the transpose launch then.
bool gemm_reads_plain_b(const Ctx* c, int64_t rows_max, int64_t a_rows, int k, int n_out, int epi)
{
    if (takes_big_kernel(c, rows_max, n_out, k, a_rows, epi)) return big_kernel_reads_plain_b(a_rows, k, n_out, epi);
    return n_out % 8 == 0 && (epi == kEpiPlain || epi == kEpiMinus);
}

bool gemm_rows_bf16(Ctx* c, const void* A, int64_t a_rows, int k, const int* row_ids, int pad_id,
                    const int* n_dev, int64_t rows_max, const void* Bt, int n_out, float* C, hipStream_t s,
                    void* H_scatter, bool caller_wants_C, int epi, const void* aux, const void* B_plain)
{
    if (rows_max <= 0) return false;
    if (takes_big_kernel(c, rows_max, n_out, k, a_rows, epi)) {
        // Fusing the gather pays when there are tiles for every CU: with a handful of tiles the
        // position stores of a tile run on one CU while a separate gather spreads over all.
        const bool fuse = H_scatter && epi == kEpiPlain;
        const ScatterArgs sc = {c->offsets, c->perm, H_scatter, (int64_t)n_out, caller_wants_C ? 1 : 0,
                               c->cfg.h_dtype == GRAM_BF16 ? 1 : 0};
        if (big_kernel_reads_plain_b(a_rows, k, n_out, epi) && B_plain)
            launch_gemm_nt(c, static_cast<const uint16_t*>(A), k, a_rows, row_ids, n_dev, rows_max,
                           static_cast<const uint16_t*>(B_plain), n_out, k, n_out, k, C, n_out, s,
                           fuse ? &sc : nullptr, pad_id, epi, aux, true);
        else
            launch_gemm_nt(c, static_cast<const uint16_t*>(A), k, a_rows, row_ids, n_dev, rows_max,
                           static_cast<const uint16_t*>(Bt), k, n_out, n_out, k, C, n_out, s, fuse ? &sc : nullptr,
                           pad_id, epi, aux);
        return fuse;
    }
    const dim3 grid((n_out + BN - 1) / BN, (unsigned)((rows_max + BM - 1) / BM));
    const uint16_t* a16 = static_cast<const uint16_t*>(A);
    const uint16_t* b16 = static_cast<const uint16_t*>(Bt);
    if (B_plain && n_out % 8 == 0 && (epi == kEpiPlain || epi == kEpiMinus)) {
        // the kernel reads the untransposed operand itself
        const uint16_t* w16 = static_cast<const uint16_t*>(B_plain);
        if (epi == kEpiMinus)
            launch(c, KID_ENCODE_BF16, k_encode_bf16<kEpiMinus, true>, grid, dim3(kBlock), s, a16, w16, row_ids,
                   n_dev, k, n_out, pad_id, C, aux);
        else
            launch(c, KID_ENCODE_BF16, k_encode_bf16<kEpiPlain, true>, grid, dim3(kBlock), s, a16, w16, row_ids,
                   n_dev, k, n_out, pad_id, C, aux);
        return false;
    }
    if (epi == kEpiReluBf16)
        launch(c, KID_ENCODE_BF16, k_encode_bf16<kEpiReluBf16>, grid, dim3(kBlock), s, a16, b16, row_ids, n_dev, k,
               n_out, pad_id, C, aux);
    else if (epi == kEpiMinus)
        launch(c, KID_ENCODE_BF16, k_encode_bf16<kEpiMinus>, grid, dim3(kBlock), s, a16, b16, row_ids, n_dev, k,
               n_out, pad_id, C, aux);
    else if (epi == kEpiGate)
        launch(c, KID_ENCODE_BF16, k_encode_bf16<kEpiGate>, grid, dim3(kBlock), s, a16, b16, row_ids, n_dev, k,
               n_out, pad_id, C, aux);
    else
        launch(c, KID_ENCODE_BF16, k_encode_bf16<kEpiPlain>, grid, dim3(kBlock), s, a16, b16, row_ids, n_dev, k,
               n_out, pad_id, C, aux);
    return false;
}

bool encode_forward(Ctx* c, const void* X, const void* W, const int* uniq, const int* u_dev,
                    int64_t rows_max, float* E, hipStream_t s, void* H_scatter, bool caller_wants_E, int epi,
                    const void* aux)
{
    if (rows_max <= 0) return false;
    const int d_in = c->cfg.d_in, d = c->cfg.d;
    if (c->cfg.xw_dtype == GRAM_BF16) {
        // both kernels can read W as it is for most shapes (no transposed copy, one launch less)
        const bool direct = gemm_reads_plain_b(c, rows_max, c->cfg.vocab_n, d_in, d, epi);
        if (!direct) transpose_weight(c, W, d_in, d, c->Wt, s);
        return gemm_rows_bf16(c, X, c->cfg.vocab_n, d_in, uniq, c->cfg.pad_id, u_dev, rows_max, c->Wt, d, E, s,
                              H_scatter, caller_wants_E, epi, aux, direct ? W : nullptr);
    }
    launch(c, KID_ENCODE_F32, k_encode_f32, dim3((d + 63) / 64, (unsigned)((rows_max + 3) / 4)),
           dim3(kBlock), s, static_cast<const float*>(X), static_cast<const float*>(W), uniq, u_dev,
           d_in, d, c->cfg.pad_id, E);
    return false;
}

// ---- weight gradient -----------------------------------------------------------
//
// The output is small (d_in x d) and the contraction runs over all rows of the
// persistent buffer, so the rows are cut into `splits` contiguous ranges
// (split-K); each range writes a float32 partial and k_wgrad_reduce adds the
// partials in range order.  The ranges depend only on the number of rows in
// the buffer, so the result is reproducible.
//
// ---- weight gradient without transposed copies ---------------------------------------
//
// dW[i,c] = sum_s X[item_s, i] * bf16(G[s, c]): both operands have the contraction
// index s (buffer row) as their slow dimension in memory.  Instead of first
// writing transposed copies, this kernel loads 32 buffer rows x 256 features of
// X (gathered through id_of_slot) and 32 x 256 columns of G per slab, rounds G
// to bf16 in registers, parks both in LDS as [s][256] rows and builds the MFMA
// fragments with the transposing LDS read of gfx950 (ds_read_b64_tr_b16): the
// 16 lanes of a group supply the addresses of a 4 (s) x 16 (m) block as 8-byte
// pieces (lane j: row j / 4, columns 4 (j % 4) .. + 3) and lane i of the group
// receives column i of the 4 rows, i.e. 4 consecutive values of the contraction
// index for one output row, which is the operand layout of
// v_mfma_f32_32x32x16_bf16 (two such reads per 8-value fragment).
// LDS rows are 512 bytes; 16-byte chunk p of row s sits at p ^ ((s & 3) << 2).  A half-wave of
// such a read is two groups, i.e. 4 rows x 4 neighbouring chunks; with the row number XOR-ed
// into bits 2-3 of the chunk index those 16 pieces land in 16 different chunk positions of the
// 256-byte bank period: every bank once (XOR-ing bits 1-2 instead left half of the banks idle
// and showed as bank conflicts in 37 % of the LDS cycles).
// Loads go through buffer descriptors; a row past the end of the buffer, a
// padding item or a column past the matrix edge is turned into an out-of-range
// offset, for which the hardware returns zeros.  WIDE (an operand beyond the 4 GiB
// of a descriptor): plain 64-bit addresses, and such a load is skipped instead.
// Same pipeline as k_gemm_nt_bf16: register-staged loads, two LDS stages, one
// barrier per slab of 32 buffer rows; split-K with one K range per XCD.
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef short v8i16 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4i16 lds_v4i16;
constexpr int WK = 32;                       // buffer rows per slab
constexpr int WROWB = 512;                   // bytes per LDS row (256 bf16)
constexpr int WOPB = WK * WROWB;             // bytes per operand and stage
constexpr int WSTAGEB = 2 * WOPB;
constexpr size_t WSMEM = 2 * (size_t)WSTAGEB;
constexpr uint32_t kOutOfRange = 0xFFFFFFF0u;
constexpr int kWgradWaves = 8;

// NW = waves per block: 4 (128x128 each) or 8 (128x64 each, two per SIMD).
// EXPORT: the end of a window also copies the buffer rows out in ascending-ID order
// (gram_flush); this kernel has every row of G in registers anyway, so it writes row s to
// G_total[rank_of_slot[s]] (rank_of_slot NULL: the buffer is in that order already) and the
// export kernel's second read of the buffer is saved.  The feature tiles that share a slab of G
// share its rows: tile f writes the rows t of a wave with t % f_tiles == f.
struct WgradExport {
    float* G_total;            // [rows held, d]
    const int* rank_of_slot;   // [rows held] or NULL
    // one-step windows: the last meta_blocks blocks of the grid export IDs and counts and clear the
    // slot map (what k_flush_meta does), so the end of such a window is two launches
    int meta_blocks;
    const long long* cnt_of_slot;
    int* slot_of;
    int* uniq_total;           // nullable
    int* counts_total;         // nullable
    int* u_total_dev;          // nullable
    int* scal;
};
template <int NW, bool WIDE = false, bool EXPORT = false>
__global__ __launch_bounds__(NW * 64) void k_wgrad_tn_bf16(
    const uint16_t* __restrict__ X, uint32_t x_bytes, const int* __restrict__ id_of_slot,
    const float* __restrict__ G, uint32_t g_bytes, const int* __restrict__ rows_dev, int d_in, int d,
    int pad_id, int splits, float* __restrict__ partial, int row_begin, int row_end, WgradExport ex)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    if (EXPORT && ex.meta_blocks > 0 && blockIdx.x >= gridDim.x - ex.meta_blocks) {
        const int n_ = *rows_dev;
        const int mb = blockIdx.x - (gridDim.x - ex.meta_blocks);
        for (int r = mb * (NW * 64) + threadIdx.x; r < n_; r += ex.meta_blocks * (NW * 64))
            flush_meta_row(r, id_of_slot, nullptr, ex.cnt_of_slot, ex.slot_of, ex.uniq_total, ex.counts_total, nullptr);
        if (mb == 0 && threadIdx.x == 0) {
            if (ex.u_total_dev) *ex.u_total_dev = n_;
            ex.scal[kSFlushN] = n_;
        }
        return;
    }
    const int tiles_c = (d + 255) / 256, tiles = ((d_in + 255) / 256) * tiles_c;
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int z = xcd + 8 * (q / tiles);
    const int i0 = ((q % tiles) / tiles_c) * 256, c0 = ((q % tiles) % tiles_c) * 256;
    if (z >= splits) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NT = NW == 4 ? 4 : 2;          // 32-column MFMA tiles per wave
    constexpr int RW = 32 / NW;                  // buffer rows of a slab this wave loads
    // two register sets for loads in flight: a load has two slabs of MFMAs to land (246 VGPRs
    // with 8 waves, so two waves per SIMD still fit)
    constexpr int SETS = 2;
    const int wm = NW == 4 ? wave >> 1 : wave >> 2, wn = NW == 4 ? wave & 1 : wave & 3;

    // buffer rows [row_begin, U) take part (row_end clips U: the chunked call); slabs stay aligned
    // to multiples of WK rows, rows outside the range are loaded as zeros
    const int rows_held = *rows_dev;
    const int U = rows_held < row_end ? rows_held : row_end;
    const int sl0 = row_begin / WK;
    const int slabs_all = U > row_begin ? (U + WK - 1) / WK - sl0 : 0;
    const int per = (slabs_all + splits - 1) / splits;
    const int sl_begin = sl0 + z * per;
    int nslab = sl0 + slabs_all - sl_begin;
    if (nslab > per) nslab = per;
    partial += (int64_t)z * d_in * d;

    const __amdgpu_buffer_rsrc_t rsX = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(X), 0, x_bytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t rsG = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(G), 0, g_bytes, kBufferFlags);

    // X loader: instruction t of wave w moves buffer rows RW w + 2 t and + 1 (lane / 32 picks the
    // row), lane % 32 = position of the 16-byte chunk in the LDS row
    const int a_row = wave * RW + (lane >> 5);                        // + 2 t
    const int a_pos = lane & 31;
    // G loader: instruction t of wave w moves buffer row RW w + t; lane l holds columns 4 l .. 4 l + 3
    const int g_col = c0 + 4 * lane;
    const bool g_col_ok = g_col < d;
    unsigned char* parkA = smem + (wave * RW) * WROWB + lane * 16;   // + t * 1024 (two rows per t)
    unsigned char* parkG = smem + WOPB + (wave * RW) * WROWB + (lane & 1) * 8;

    f32x16 acc[4][NT];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // fragment addresses (see the header comment): group g = lane / 16, j = lane % 16
    const int j16 = lane & 15, grp = lane >> 4;
    const int f_row = (grp >> 1) * 8 + (j16 >> 2);                   // + 16 ks + 4 h
    const int f_x = ((j16 >> 2) & 3) << 2;
    // chunk index within the whole 512-byte row (the swizzle acts on it): the wave's quadrant starts
    // at chunk 16 wm (A) / NT 4 wn (B)
    int f_offA[4], f_offB[NT];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        f_offA[i] = f_row * WROWB + (((wm * 16 + i * 4 + (grp & 1) * 2 + ((j16 & 3) >> 1)) ^ f_x) * 16) + (j16 & 1) * 8;
#pragma unroll
    for (int i = 0; i < NT; ++i)
        f_offB[i] = WOPB + f_row * WROWB +
                    (((wn * (NT * 4) + i * 4 + (grp & 1) * 2 + ((j16 & 3) >> 1)) ^ f_x) * 16) + (j16 & 1) * 8;

    bf16x8 fa[2][4], fb[2][NT];
    v4i32 ra[SETS][RW / 2], rg[SETS][RW];
    // (EXPORT) rk[set]: lane t < RW holds the output row of the t-th buffer row of the slab in that
    // set, -1 if the row is not to be written; fetched BEFORE the slab's data loads (see below)
    int rk[EXPORT ? SETS : 1];
    bool ex_mine[RW];
    {
        const int f_tiles = (d_in + 255) / 256, f_idx = i0 / 256;
#pragma unroll
        for (int t = 0; t < RW; ++t) ex_mine[t] = EXPORT && (t % f_tiles) == f_idx;
    }
    // item IDs: ids_next receives the load for the slab after next, ids_cur holds the ones the next
    // data loads use.  The ID load is issued BEFORE the data loads of an iteration: memory operations
    // return in order, so waiting for an ID load that was issued after them would drain them all
    // and leave a single slab of loads in flight.
    int ids_next[RW / 2], ids_cur[RW / 2];

#define GRAM_TR(PTR) __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(PTR))
#define GRAM_FRAGS(FS, STAGE, KS)                                                                   \
    {                                                                                               \
        const unsigned char* sb_ = smem + (STAGE) * WSTAGEB + (KS) * 16 * WROWB;                    \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                             \
            const v4i16 a0 = GRAM_TR(sb_ + f_offA[i]);                                       \
            const v4i16 a1 = GRAM_TR(sb_ + f_offA[i] + 4 * WROWB);                           \
            fa[FS][i] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7)); \
        }                                                                                           \
        _Pragma("unroll") for (int i = 0; i < NT; ++i) {                                            \
            const v4i16 b0 = GRAM_TR(sb_ + f_offB[i]);                                       \
            const v4i16 b1 = GRAM_TR(sb_ + f_offB[i] + 4 * WROWB);                           \
            fb[FS][i] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7)); \
        }                                                                                           \
    }
    // (Raising the wave priority around the fragment reads and MFMAs of a k-step paid while a
    // single slab of loads was in flight; with two it costs 4 %.)
#define GRAM_MMA(FS)                                                                                \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                   \
        _Pragma("unroll") for (int j = 0; j < NT; ++j)                                              \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[FS][i], fb[FS][j], acc[i][j], 0, 0, 0);
    // item IDs of the X rows this lane will fetch for slab SLAB (clamped: a slab past the end is
    // loaded but never multiplied)
#define GRAM_IDS(SLAB)                                                                              \
    {                                                                                               \
        const int sb_ = (sl_begin + ((SLAB) < last ? (SLAB) : last)) * WK;                          \
        _Pragma("unroll") for (int t = 0; t < RW / 2; ++t) {                                        \
            const int slot = sb_ + a_row + 2 * t;                                                   \
            ids_next[t] = (slot < U && slot >= row_begin) ? (id_of_slot ? id_of_slot[slot] : slot) : pad_id; \
        }                                                                                           \
    }
#define GRAM_IDS_TAKE                                                                               \
    _Pragma("unroll") for (int t = 0; t < RW / 2; ++t) ids_cur[t] = ids_next[t];
#define GRAM_LOAD(SET, SLAB)                                                                        \
    {                                                                                               \
        const int sb_ = (sl_begin + ((SLAB) < last ? (SLAB) : last)) * WK;                          \
        if (EXPORT) {                                                                               \
            const int slot = sb_ + wave * RW + lane;                                                \
            const bool okr = lane < RW && slot < U && slot >= row_begin;                            \
            rk[(SET) % SETS] = okr ? (ex.rank_of_slot ? ex.rank_of_slot[slot] : slot) : -1;         \
        }                                                                                           \
        _Pragma("unroll") for (int t = 0; t < RW / 2; ++t) {                                        \
            const int kk = a_row + 2 * t;                                                           \
            const int feat = i0 + ((a_pos ^ ((kk & 3) << 2)) * 8);                                  \
            const int id = ids_cur[t];                                                              \
            const bool ok = id != pad_id && feat < d_in && sb_ + kk < U && sb_ + kk >= row_begin;   \
            if (WIDE) {                                                                             \
                v4i32 v_ = {0, 0, 0, 0};                                                            \
                if (ok) v_ = *reinterpret_cast<const v4i32*>(X + (int64_t)id * d_in + feat);        \
                ra[(SET) % SETS][t] = v_;                                                           \
            } else {                                                                                \
                const uint32_t off = ok ? (uint32_t)(((int64_t)id * d_in + feat) * 2) : kOutOfRange; \
                ra[(SET) % SETS][t] = __builtin_amdgcn_raw_buffer_load_b128(rsX, off, 0, 0);        \
            }                                                                                       \
        }                                                                                           \
        _Pragma("unroll") for (int t = 0; t < RW; ++t) {                                            \
            const int slot = sb_ + wave * RW + t;                                                    \
            const bool okg = g_col_ok && slot < U && slot >= row_begin;                             \
            if (WIDE) {                                                                             \
                v4i32 v_ = {0, 0, 0, 0};                                                            \
                if (okg) v_ = *reinterpret_cast<const v4i32*>(G + (int64_t)slot * d + g_col);       \
                rg[(SET) % SETS][t] = v_;                                                           \
            } else {                                                                                \
                const uint32_t off = okg ? (uint32_t)(((int64_t)slot * d + g_col) * 4) : kOutOfRange; \
                rg[(SET) % SETS][t] = __builtin_amdgcn_raw_buffer_load_b128(rsG, off, 0, 0);        \
            }                                                                                       \
        }                                                                                           \
    }
#define GRAM_PARK(SET, STAGE)                                                                       \
    {                                                                                               \
        unsigned char* pa_ = parkA + (STAGE) * WSTAGEB;                                             \
        unsigned char* pg_ = parkG + (STAGE) * WSTAGEB;                                             \
        _Pragma("unroll") for (int t = 0; t < RW / 2; ++t)                                          \
            *reinterpret_cast<v4i32*>(pa_ + t * 1024) = ra[(SET) % SETS][t];                                 \
        _Pragma("unroll") for (int t = 0; t < RW; ++t) {                                            \
            const v4i32 v = rg[(SET) % SETS][t];                                                             \
            const uint32_t lo = pack_bf16x2(__int_as_float(v.x), __int_as_float(v.y));              \
            const uint32_t hi = pack_bf16x2(__int_as_float(v.z), __int_as_float(v.w));              \
            const int pos = (lane >> 1) ^ ((t & 3) << 2);        /* row RW w + t: (row & 3) == (t & 3) */ \
            *reinterpret_cast<uint2*>(pg_ + t * WROWB + pos * 16) = make_uint2(lo, hi);             \
            if (EXPORT && ex_mine[t]) {                                                             \
                const int r_ = __builtin_amdgcn_readlane(rk[(SET) % SETS], t);                      \
                if (r_ >= 0 && g_col_ok)                                                            \
                    __builtin_nontemporal_store(v, reinterpret_cast<v4i32*>(ex.G_total + (int64_t)r_ * d + g_col)); \
            }                                                                                       \
        }                                                                                           \
    }
    // (fixed interleaving patterns measured slower here than the compiler's own order)
#define GRAM_ITER(SL, P)                                                                            \
    {                                                                                               \
        GRAM_FRAGS(1, (SL) & 1, 1)                                                                  \
        GRAM_MMA(0)                                                                                 \
        GRAM_PARK(P, ((SL) + 1) & 1)                                                                \
        __syncthreads();                                                                            \
        GRAM_IDS_TAKE                                                                               \
        GRAM_IDS((SL) + 2 + SETS)                                                                   \
        GRAM_LOAD(P, (SL) + 1 + SETS)                                                               \
        GRAM_FRAGS(0, ((SL) + 1) & 1, 0)                                                            \
        GRAM_MMA(1)                                                                                 \
    }

    if (nslab > 0) {
        const int last = nslab - 1;
        GRAM_IDS(0)
        GRAM_IDS_TAKE
        GRAM_IDS(1)
        GRAM_LOAD(0, 0)
        GRAM_IDS_TAKE
        GRAM_IDS(2)
        GRAM_LOAD(1, 1)
        GRAM_PARK(0, 0)
        GRAM_IDS_TAKE
        GRAM_IDS(SETS + 1)
        GRAM_LOAD(0, SETS)
        __syncthreads();
        GRAM_FRAGS(0, 0, 0)
        int sl = 0;
        for (; sl + 1 < last; sl += 2) {
            GRAM_ITER(sl, 1)          // set 1 holds slab sl+1, set 0 holds slab sl+2
            GRAM_ITER(sl + 1, 0)
        }
        if (sl < last) GRAM_ITER(sl, 1)
        GRAM_FRAGS(1, last & 1, 1)
        GRAM_MMA(0)
        GRAM_MMA(1)
    }

    // accumulator element r of a lane sits at (row, col) = ((r / 4) * 8 + (lane / 32) * 4 + r % 4, lane % 32)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int fi = i0 + wm * 128 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            if (fi < d_in) {
                float* row = partial + (int64_t)fi * d + c0 + wn * (NT * 32) + (lane & 31);
#pragma unroll
                for (int jj = 0; jj < NT; ++jj)
                    if (c0 + wn * (NT * 32) + jj * 32 + (lane & 31) < d) row[jj * 32] = acc[i][jj][r];
            }
        }
}
#undef GRAM_TR
#undef GRAM_FRAGS
#undef GRAM_MMA
#undef GRAM_IDS
#undef GRAM_IDS_TAKE
#undef GRAM_LOAD
#undef GRAM_PARK
#undef GRAM_ITER

__device__ __forceinline__ void split_range(int u_total, int splits, int z, int* kb, int* ke)
{
    const int chunk = (u_total + splits - 1) / splits;
    const int b = z * chunk;
    int e = b + chunk;
    if (e > u_total) e = u_total;
    *kb = b < u_total ? b : u_total;
    *ke = e < *kb ? *kb : e;
}

__global__ __launch_bounds__(kBlock) void k_wgrad_f32(
    const float* __restrict__ X, const int* __restrict__ id_of_slot, const float* __restrict__ G,
    const int* __restrict__ rows_dev, int d_in, int d, int pad_id, int splits,
    float* __restrict__ partial, int row_begin, int row_end)
{
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int i = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int z = blockIdx.z;
    if (i >= d_in || c >= d) return;
    int kb, ke;
    const int rows_held = *rows_dev;
    const int u_end = rows_held < row_end ? rows_held : row_end;
    split_range(u_end > row_begin ? u_end - row_begin : 0, splits, z, &kb, &ke);
    kb += row_begin;
    ke += row_begin;
    float acc = 0.f;
    for (int sidx = kb; sidx < ke; ++sidx) {
        const int id = id_of_slot ? id_of_slot[sidx] : sidx;
        if (id != pad_id) acc = fmaf(X[(int64_t)id * d_in + i], G[(int64_t)sidx * d + c], acc);
    }
    partial[((int64_t)z * d_in + i) * d + c] = acc;
}

__global__ __launch_bounds__(kBlock) void k_wgrad_reduce(const float4* __restrict__ partial,
                                                         int64_t n4, int splits,
                                                         float4* __restrict__ dW, int accumulate)
{
    const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= n4) return;
    float4 acc = accumulate ? dW[e] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
    for (int z = 0; z < splits; ++z) {
        const float4 v = partial[(int64_t)z * n4 + e];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    dW[e] = acc;
}

int wgrad_splits_for(const gram_config& cfg)
{
    return wgrad_splits_dims(cfg.d_in, cfg.d, cfg.xw_dtype == GRAM_BF16);
}

int wgrad_splits_dims(int d_in, int d, bool bf16)
{
    if (!bf16) return 4;
    const int tiles = ((d_in + TM - 1) / TM) * ((d + TN - 1) / TN);
    int s = 256 / tiles / 8 * 8;      // one block per CU; a multiple of 8 (one K range per XCD)
    if (s < 8) s = 8;
    if (s > 64) s = 64;
    return s;
}

bool encoder_wgrad(Ctx* c, const void* X, float* dW, hipStream_t s, int64_t first_row, int64_t n_rows,
                   bool accumulate, const WgradRows* other, float* export_G, const int* rank_of_slot,
                   const WindowMeta* meta)
{
    bool exported = false;
    const int d_in = other && other->d_in ? other->d_in : c->cfg.d_in;
    const int d = other && other->d ? other->d : c->cfg.d;
    const int64_t x_rows = other && other->x_rows ? other->x_rows : c->cfg.vocab_n;
    const int pad_id = other && other->d_in ? other->pad_id : c->cfg.pad_id;
    int S = other && other->d_in ? wgrad_splits_dims(d_in, d, c->cfg.xw_dtype == GRAM_BF16) : c->wg_splits;
    // the rows contracted over: the persistent buffer (id_of_slot is NULL for the dense layout:
    // the item of row r is r), or the caller's (ids, rows) pairs
    const int64_t cap = other ? other->n_max : c->cap_total;
    const int* ids = other ? other->ids : c->id_of_slot;
    const float* rows = other ? other->rows : c->G;
    const int* rows_dev = other ? other->n_dev : c->scal + kSUTotal;
    const int row_begin = (int)(first_row < cap ? first_row : cap);
    const int row_end = (int)(n_rows < cap - row_begin ? row_begin + n_rows : cap);
    if (c->cfg.xw_dtype == GRAM_BF16) {
        // a short window does not need all the ranges: at least 8 slabs of 32 buffer rows each
        // (from the host's bound on the rows in the buffer), still a multiple of 8
        int64_t rows_bound = (other || c->dense) ? cap : (c->window_positions < cap ? c->window_positions : cap);
        if (rows_bound > row_end - row_begin) rows_bound = row_end - row_begin;
        const int64_t slabs_bound = rows_bound / TK + 1;
        int64_t want = slabs_bound / 8 / 8 * 8;
        if (want < 8) want = 8;
        if (want < S) S = (int)want;
        const int64_t x_bytes = x_rows * d_in * 2, g_bytes = cap * d * 4;
        const int tiles = ((d_in + 255) / 256) * ((d + 255) / 256);
        const WgradExport no_export = {nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
        if (x_bytes < kBufferWindow && g_bytes < kBufferWindow && export_G && !other) {
            constexpr auto kern = k_wgrad_tn_bf16<kWgradWaves, false, true>;
            ensure_dynamic_lds<kern>((int)WSMEM);
            WgradExport ex = no_export;
            ex.G_total = export_G;
            ex.rank_of_slot = rank_of_slot;
            if (meta) {
                int64_t mb = (rows_bound + kWgradWaves * 64 - 1) / (kWgradWaves * 64);
                ex.meta_blocks = (int)(mb < 1 ? 1 : (mb > 64 ? 64 : mb));
                ex.cnt_of_slot = c->cnt_of_slot;
                ex.slot_of = c->slot_of;
                ex.uniq_total = meta->uniq_total;
                ex.counts_total = meta->counts_total;
                ex.u_total_dev = meta->u_total_dev;
                ex.scal = c->scal;
            }
            launch_smem(c, KID_WGRAD_BF16, kern, dim3((unsigned)(tiles * S + ex.meta_blocks)), dim3(kWgradWaves * 64), WSMEM, s,
                        static_cast<const uint16_t*>(X), (uint32_t)x_bytes, ids, rows, (uint32_t)g_bytes,
                        rows_dev, d_in, d, pad_id, S, c->wg_partial, row_begin, row_end, ex);
            exported = true;
        } else if (x_bytes < kBufferWindow && g_bytes < kBufferWindow) {
            constexpr auto kern = k_wgrad_tn_bf16<kWgradWaves, false>;
            ensure_dynamic_lds<kern>((int)WSMEM);
            launch_smem(c, KID_WGRAD_BF16, kern, dim3((unsigned)(tiles * S)), dim3(kWgradWaves * 64), WSMEM, s,
                        static_cast<const uint16_t*>(X), (uint32_t)x_bytes, ids, rows, (uint32_t)g_bytes,
                        rows_dev, d_in, d, pad_id, S, c->wg_partial, row_begin, row_end, no_export);
        } else {
            constexpr auto kern = k_wgrad_tn_bf16<kWgradWaves, true>;
            ensure_dynamic_lds<kern>((int)WSMEM);
            launch_smem(c, KID_WGRAD_BF16_WIDE, kern, dim3((unsigned)(tiles * S)), dim3(kWgradWaves * 64), WSMEM, s,
                        static_cast<const uint16_t*>(X), 0u, ids, rows, 0u, rows_dev, d_in, d, pad_id, S,
                        c->wg_partial, row_begin, row_end, no_export);
        }
    } else {
        launch(c, KID_WGRAD_F32, k_wgrad_f32, dim3((d + 63) / 64, (d_in + 3) / 4, S), dim3(kBlock), s,
               static_cast<const float*>(X), ids, rows, rows_dev, d_in, d, pad_id, S,
               c->wg_partial, row_begin, row_end);
    }
    const int64_t n4 = (int64_t)d_in * d / 4;
    launch(c, KID_WGRAD_REDUCE, k_wgrad_reduce, dim3((unsigned)((n4 + kBlock - 1) / kBlock)), dim3(kBlock), s,
           reinterpret_cast<const float4*>(c->wg_partial), n4, S, reinterpret_cast<float4*>(dW), accumulate ? 1 : 0);
    return exported;
}

}  // namespace gram
