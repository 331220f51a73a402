// The two dense contractions of the GRAM step, with the dense linear stand-in
// for the content encoder:
//   forward  (Algorithm 1 step 1, Eq. 4):  E[j,:]  = X[uniq[j],:] . W
//   wgrad    (Algorithm 1 step 4, Eq. 7/9): dW[i,c] = sum_s X[item_s, i] * G[s, c]
// bf16 inputs run on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulate); the float32 variant is plain FMA code for small problems.
// Rows of X are gathered through the ID list inside the tile loads, so the
// unique items' features are never copied.
#include "gram_internal.h"

namespace gram {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDS_STRIDE = BK + 8;   // bf16 elements per LDS row (80 bytes: 16-byte aligned, staggers banks)

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// One BK slab of a 128x128 block tile: each of the 4 waves owns a 64x64
// quadrant as 2x2 MFMA tiles.  sA/sB hold [row][k] with k contiguous.
__device__ __forceinline__ void mma_slab(const uint16_t* sA, const uint16_t* sB, int wm, int wn,
                                         int lane, f32x16 (&acc)[2][2])
{
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
        const int koff = ks * 16 + (lane >> 5) * 8;
        bf16x8 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            a[i] = *reinterpret_cast<const bf16x8*>(&sA[(wm * 64 + i * 32 + (lane & 31)) * LDS_STRIDE + koff]);
            b[i] = *reinterpret_cast<const bf16x8*>(&sB[(wn * 64 + i * 32 + (lane & 31)) * LDS_STRIDE + koff]);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

// Accumulator element r of lane `lane` in a 32x32 MFMA tile sits at
// (row, col) = ((r / 4) * 8 + (lane / 32) * 4 + r % 4, lane % 32).
template <typename F>
__device__ __forceinline__ void for_each_acc(const f32x16 (&acc)[2][2], int wm, int wn, int lane, F f)
{
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * 64 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                const int col = wn * 64 + j * 32 + (lane & 31);
                f(row, col, acc[i][j][r]);
            }
}

// ---- W[d_in,d] -> Wt[d,d_in] (bf16) ----------------------------------------

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

// ---- forward, bf16 -----------------------------------------------------------

__global__ __launch_bounds__(kBlock) void k_encode_bf16(
    const uint16_t* __restrict__ X, const uint16_t* __restrict__ Wt, const int* __restrict__ uniq,
    const int* __restrict__ u_dev, int d_in, int d, int pad_id, float* __restrict__ E)
{
    __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LDS_STRIDE];
    const int U = *u_dev;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    if (m0 >= U) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // each thread moves two 16-byte chunks of A and of B per slab
    const uint16_t* pa[2];
    const uint16_t* pb[2];
    int kc[2], lrow[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int cid = tid + h * kBlock;
        lrow[h] = cid >> 2;
        kc[h] = (cid & 3) * 8;
        const int j = m0 + lrow[h];
        pa[h] = j < U ? X + (int64_t)uniq[j] * d_in : nullptr;
        pb[h] = n0 + lrow[h] < d ? Wt + (int64_t)(n0 + lrow[h]) * d_in : nullptr;
    }
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    uint4 ra[2], rb[2];
    auto load_slab = [&](int k0) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const bool kin = k0 + kc[h] < d_in;
            ra[h] = (pa[h] && kin) ? *reinterpret_cast<const uint4*>(pa[h] + k0 + kc[h]) : zero4;
            rb[h] = (pb[h] && kin) ? *reinterpret_cast<const uint4*>(pb[h] + k0 + kc[h]) : zero4;
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    load_slab(0);
    for (int k0 = 0; k0 < d_in; k0 += BK) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            *reinterpret_cast<uint4*>(&sA[lrow[h] * LDS_STRIDE + kc[h]]) = ra[h];
            *reinterpret_cast<uint4*>(&sB[lrow[h] * LDS_STRIDE + kc[h]]) = rb[h];
        }
        __syncthreads();
        if (k0 + BK < d_in) load_slab(k0 + BK);
        mma_slab(sA, sB, wm, wn, lane, acc);
        __syncthreads();
    }

    for_each_acc(acc, wm, wn, lane, [&](int row, int col, float v) {
        const int j = m0 + row, c = n0 + col;
        if (j < U && c < d) E[(int64_t)j * d + c] = uniq[j] == pad_id ? 0.f : v;
    });
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

void encode_forward(Ctx* c, const void* X, const void* W, const int* uniq, const int* u_dev,
                    int64_t rows_max, float* E, hipStream_t s)
{
    if (rows_max <= 0) return;
    const int d_in = c->cfg.d_in, d = c->cfg.d;
    if (c->cfg.xw_dtype == GRAM_BF16) {
        launch(c, KID_TRANSPOSE_U16, k_transpose_u16, dim3((d + 31) / 32, (d_in + 31) / 32), dim3(kBlock), s,
                           static_cast<const uint16_t*>(W), d_in, d, static_cast<uint16_t*>(c->Wt));
        launch(c, KID_ENCODE_BF16, k_encode_bf16, dim3((d + BN - 1) / BN, (unsigned)((rows_max + BM - 1) / BM)),
                           dim3(kBlock), s, static_cast<const uint16_t*>(X),
                           static_cast<const uint16_t*>(c->Wt), uniq, u_dev, d_in, d, c->cfg.pad_id, E);
    } else {
        launch(c, KID_ENCODE_F32, k_encode_f32, dim3((d + 63) / 64, (unsigned)((rows_max + 3) / 4)),
                           dim3(kBlock), s, static_cast<const float*>(X),
                           static_cast<const float*>(W), uniq, u_dev, d_in, d, c->cfg.pad_id, E);
    }
}

// ---- weight gradient -----------------------------------------------------------
//
// The output is small (d_in x d) and the contraction runs over all buffer rows,
// so the rows are split into `splits` contiguous ranges (split-K); each range
// writes a float32 partial and k_wgrad_reduce adds the partials in range
// order.  The ranges depend only on the number of rows in the buffer.

__device__ __forceinline__ void split_range(int u_total, int splits, int z, int align, int* kb, int* ke)
{
    int chunk = (u_total + splits - 1) / splits;
    chunk = (chunk + align - 1) / align * align;
    const int b = z * chunk;
    int e = b + chunk;
    if (e > u_total) e = u_total;
    *kb = b < u_total ? b : u_total;
    *ke = e < *kb ? *kb : e;
}

__global__ __launch_bounds__(kBlock) void k_wgrad_bf16(
    const uint16_t* __restrict__ X, const int* __restrict__ id_of_slot, const float* __restrict__ G,
    const int* __restrict__ scal, int d_in, int d, int pad_id, int splits,
    float* __restrict__ partial)
{
    __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LDS_STRIDE];   // [i][slot]
    __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LDS_STRIDE];   // [c][slot]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i0 = blockIdx.y * BM, n0 = blockIdx.x * BN, z = blockIdx.z;
    int kb, ke;
    split_range(scal[kSUTotal], splits, z, BK, &kb, &ke);

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    for (int k0 = kb; k0 < ke; k0 += BK) {
        // A: 32 buffer rows x 128 features, 16 bytes (8 features) per chunk, stored transposed
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int cid = tid + h * kBlock;
            const int kk = cid >> 4, ic = (cid & 15) * 8;
            uint4 v = zero4;
            if (k0 + kk < ke && i0 + ic < d_in) {
                const int id = id_of_slot[k0 + kk];
                if (id != pad_id) v = *reinterpret_cast<const uint4*>(X + (int64_t)id * d_in + i0 + ic);
            }
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                sA[(ic + e) * LDS_STRIDE + kk] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
        }
        // B: 32 buffer rows x 128 columns of G (float32), rounded to bf16, stored transposed
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const int cid = tid + h * kBlock;
            const int kk = cid >> 5, cc = (cid & 31) * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k0 + kk < ke && n0 + cc < d)
                v = *reinterpret_cast<const float4*>(G + (int64_t)(k0 + kk) * d + n0 + cc);
            sB[(cc + 0) * LDS_STRIDE + kk] = f32_to_bf16_rne(v.x);
            sB[(cc + 1) * LDS_STRIDE + kk] = f32_to_bf16_rne(v.y);
            sB[(cc + 2) * LDS_STRIDE + kk] = f32_to_bf16_rne(v.z);
            sB[(cc + 3) * LDS_STRIDE + kk] = f32_to_bf16_rne(v.w);
        }
        __syncthreads();
        mma_slab(sA, sB, wm, wn, lane, acc);
        __syncthreads();
    }

    float* out = partial + (int64_t)z * d_in * d;
    for_each_acc(acc, wm, wn, lane, [&](int row, int col, float v) {
        const int i = i0 + row, c = n0 + col;
        if (i < d_in && c < d) out[(int64_t)i * d + c] = v;
    });
}

__global__ __launch_bounds__(kBlock) void k_wgrad_f32(
    const float* __restrict__ X, const int* __restrict__ id_of_slot, const float* __restrict__ G,
    const int* __restrict__ scal, int d_in, int d, int pad_id, int splits,
    float* __restrict__ partial)
{
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int i = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int z = blockIdx.z;
    if (i >= d_in || c >= d) return;
    int kb, ke;
    split_range(scal[kSUTotal], splits, z, 1, &kb, &ke);
    float acc = 0.f;
    for (int sidx = kb; sidx < ke; ++sidx) {
        const int id = id_of_slot[sidx];
        if (id != pad_id) acc = fmaf(X[(int64_t)id * d_in + i], G[(int64_t)sidx * d + c], acc);
    }
    partial[((int64_t)z * d_in + i) * d + c] = acc;
}

__global__ __launch_bounds__(kBlock) void k_wgrad_reduce(const float4* __restrict__ partial,
                                                         int64_t n4, int splits,
                                                         float4* __restrict__ dW)
{
    const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= n4) return;
    float4 acc = partial[e];
    for (int z = 1; z < splits; ++z) {
        const float4 v = partial[(int64_t)z * n4 + e];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    dW[e] = acc;
}

int wgrad_splits_for(const gram_config& cfg)
{
    if (cfg.xw_dtype != GRAM_BF16) return 4;
    const int tiles = ((cfg.d_in + BM - 1) / BM) * ((cfg.d + BN - 1) / BN);
    int s = 512 / tiles;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return s;
}

void encoder_wgrad(Ctx* c, const void* X, float* dW, hipStream_t s)
{
    const int d_in = c->cfg.d_in, d = c->cfg.d, S = c->wg_splits;
    if (c->cfg.xw_dtype == GRAM_BF16)
        launch(c, KID_WGRAD_BF16, k_wgrad_bf16, dim3((d + BN - 1) / BN, (d_in + BM - 1) / BM, S), dim3(kBlock),
                           s, static_cast<const uint16_t*>(X), c->id_of_slot, c->G, c->scal, d_in, d,
                           c->cfg.pad_id, S, c->wg_partial);
    else
        launch(c, KID_WGRAD_F32, k_wgrad_f32, dim3((d + 63) / 64, (d_in + 3) / 4, S), dim3(kBlock), s,
                           static_cast<const float*>(X), c->id_of_slot, c->G, c->scal, d_in, d,
                           c->cfg.pad_id, S, c->wg_partial);
    const int64_t n4 = (int64_t)d_in * d / 4;
    launch(c, KID_WGRAD_REDUCE, k_wgrad_reduce, dim3((unsigned)((n4 + kBlock - 1) / kBlock)), dim3(kBlock), s,
                       reinterpret_cast<const float4*>(c->wg_partial), n4, S,
                       reinterpret_cast<float4*>(dW));
}

}  // namespace gram
