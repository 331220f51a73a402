// HBM-bound kernels of the GRAM step: row gather of representations to
// interaction positions (Algorithm 1 step 1, second half; for large batches the
// contraction in gram_gemm.hip does most of it and only the copy for very
// popular items runs here), the pseudo-targets of step 3 (Eq. 6), the
// deterministic per-item reduction of dL/dH (step 3, Eq. 6) into the buffer
// that persists over a Multi-step window (Section 4.2), and the export of that
// buffer at the end of the window.
//
// No float atomics anywhere: each buffer row has exactly one writer and a
// fixed order of additions, so results are bit-identical from run to run.
#include "gram_internal.h"

namespace gram {

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

__device__ __forceinline__ int wave_incl_scan(int v)
{
    const int lane = lane_id();
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        int t = __shfl_up(v, o);
        if (lane >= o) v += t;
    }
    return v;
}

template <int NWAVES = kWavesPerBlock>
__device__ __forceinline__ int block_excl_scan(int v, int* total, int* sm /*[NWAVES]*/)
{
    const int incl = wave_incl_scan(v);
    if (lane_id() == kWave - 1) sm[wave_id()] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) {
        const int t = sm[w];
        if (w < wave_id()) base += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return base + incl - v;
}

__device__ __forceinline__ int block_sum(int v, int* sm)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_down(v, o);
    if (lane_id() == 0) sm[wave_id()] = v;
    __syncthreads();
    int tot = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) tot += sm[w];
    __syncthreads();
    return tot;
}

__device__ __forceinline__ float4 f4_add(float4 a, float4 b)
{
    return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w);
}

// ---- fill ------------------------------------------------------------------

__global__ __launch_bounds__(kBlock) void k_fill_i32(int* __restrict__ p, int64_t n, int v)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock)
        p[i] = v;
}

void fill_i32(int* p, int64_t n, int v, hipStream_t s)
{
    if (n <= 0) return;
    int64_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_fill_i32, dim3((unsigned)blocks), dim3(kBlock), 0, s, p, n, v);
}

__global__ __launch_bounds__(kBlock) void k_iota_i32(int* __restrict__ p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock)
        p[i] = (int)i;
}

void iota_i32(int* p, int64_t n, hipStream_t s)
{
    if (n <= 0) return;
    int64_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_iota_i32, dim3((unsigned)blocks), dim3(kBlock), 0, s, p, n);
}

// ---- gather: H[p,:] = E[inverse[p],:] ---------------------------------------

// A block copies `rows_per_block` consecutive positions (about 32 KiB), so its
// writes to H form one contiguous stream; each thread keeps kGatherUnroll
// independent 16-byte loads in flight.  H is written once and not re-read here,
// so its stores bypass the caches; rows of E are re-read (once per occurrence)
// and keep ordinary cached loads, which measured faster than streaming ones.
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kGatherUnroll = 8;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// One group of 4 columns of a row of H: float32 as it is, or rounded to bf16 (HB).
template <bool HB>
__device__ __forceinline__ void store_h4(void* __restrict__ H, int64_t group, f32x4 v)
{
    if (HB) {
        const u32x2 h = {pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
        __builtin_nontemporal_store(h, static_cast<u32x2*>(H) + group);
    } else {
        __builtin_nontemporal_store(v, static_cast<f32x4*>(H) + group);
    }
}

template <bool HB>
__global__ __launch_bounds__(kBlock) void k_gather_rows(const f32x4* __restrict__ E,
                                                        const int* __restrict__ inverse, int64_t m,
                                                        int cols4, void* __restrict__ H,
                                                        int rows_per_block)
{
    const int64_t p0 = (int64_t)blockIdx.x * rows_per_block;
    const int rows = (int)(p0 + rows_per_block < m ? rows_per_block : m - p0);
    const int total = rows * cols4;
    for (int e0 = 0; e0 < total; e0 += kBlock * kGatherUnroll) {
        if (e0 + kBlock * kGatherUnroll <= total) {
            // a whole group: nothing is conditional, so the loads go out together and every store
            // waits for its own load only (with conditions around them each store waited for all
            // memory operations before it, the earlier stores included)
            int64_t src[kGatherUnroll];
#pragma unroll
            for (int u = 0; u < kGatherUnroll; ++u) {
                const int e = e0 + u * kBlock + threadIdx.x;
                const int row = e / cols4;
                src[u] = (int64_t)inverse[p0 + row] * cols4 + (e - row * cols4);
            }
            f32x4 v[kGatherUnroll];
#pragma unroll
            for (int u = 0; u < kGatherUnroll; ++u) v[u] = E[src[u]];
#pragma unroll
            for (int u = 0; u < kGatherUnroll; ++u)
                store_h4<HB>(H, p0 * cols4 + e0 + u * kBlock + threadIdx.x, v[u]);
            continue;
        }
        int64_t src[kGatherUnroll];
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u) {
            const int e = e0 + u * kBlock + threadIdx.x;
            const int row = e / cols4;
            src[u] = e < total ? (int64_t)inverse[p0 + row] * cols4 + (e - row * cols4) : -1;
        }
        f32x4 v[kGatherUnroll];
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u)
            if (src[u] >= 0) v[u] = E[src[u]];
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u)
            if (src[u] >= 0) store_h4<HB>(H, p0 * cols4 + e0 + u * kBlock + threadIdx.x, v[u]);
    }
}

void gather_rows(Ctx* c, const float* E, const int* inverse, int64_t m, void* H, hipStream_t s)
{
    if (m == 0) return;
    const int cols4 = c->cfg.d / 4;
    int rows_per_block = (kGatherUnroll * kBlock + cols4 - 1) / cols4;
    if (rows_per_block < 1) rows_per_block = 1;
    const int64_t blocks = (m + rows_per_block - 1) / rows_per_block;
    if (c->cfg.h_dtype == GRAM_BF16)
        launch(c, KID_GATHER_ROWS, k_gather_rows<true>, dim3((unsigned)blocks), dim3(kBlock), s,
               reinterpret_cast<const f32x4*>(E), inverse, m, cols4, H, rows_per_block);
    else
        launch(c, KID_GATHER_ROWS, k_gather_rows<false>, dim3((unsigned)blocks), dim3(kBlock), s,
               reinterpret_cast<const f32x4*>(E), inverse, m, cols4, H, rows_per_block);
}

// Second half of the fused forward: items with more than kLightMax positions were written to
// E only; their rows are copied to their positions here.  Blocks walk the SORTED order (all
// positions of an item adjacent), 64 rows each, and leave at once when none of their rows
// belongs to such an item, so the row of E being copied stays in cache across many blocks.
template <bool HB>
__global__ __launch_bounds__(kBlock) void k_gather_heavy(const f32x4* __restrict__ E,
                                                         const int* __restrict__ seg_of_row,
                                                         const int* __restrict__ offsets,
                                                         const int* __restrict__ perm, int64_t m,
                                                         int cols4, void* __restrict__ H,
                                                         int rows_per_block)
{
    __shared__ int s_src[64], s_dst[64];
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int rows = (int)(r0 + rows_per_block < m ? rows_per_block : m - r0);
    int heavy = 0;
    if ((int)threadIdx.x < rows) {
        const int j = seg_of_row[r0 + threadIdx.x];
        heavy = offsets[j + 1] - offsets[j] > kLightMax;
        s_src[threadIdx.x] = heavy ? j : -1;
        s_dst[threadIdx.x] = perm[r0 + threadIdx.x];
    }
    if (!__syncthreads_or(heavy)) return;
    // consecutive sorted rows mostly belong to one item: its row of E is loaded once and kept in
    // registers while it is stored to position after position
    for (int cp = threadIdx.x; cp < cols4; cp += kBlock) {
        int cur = -1;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        for (int row = 0; row < rows; ++row) {
            const int j = s_src[row];
            if (j < 0) continue;
            if (j != cur) {
                v = E[(int64_t)j * cols4 + cp];
                cur = j;
            }
            store_h4<HB>(H, (int64_t)s_dst[row] * cols4 + cp, v);
        }
    }
}

void gather_heavy(Ctx* c, const float* E, int64_t m, void* H, hipStream_t s)
{
    if (m == 0) return;
    const int cols4 = c->cfg.d / 4;
    const int rows_per_block = 64;      // the size of the kernel's row tables
    const int64_t blocks = (m + rows_per_block - 1) / rows_per_block;
    if (c->cfg.h_dtype == GRAM_BF16)
        launch(c, KID_GATHER_HEAVY, k_gather_heavy<true>, dim3((unsigned)blocks), dim3(kBlock), s,
               reinterpret_cast<const f32x4*>(E), c->seg_of_row, c->offsets, c->perm, m, cols4, H, rows_per_block);
    else
        launch(c, KID_GATHER_HEAVY, k_gather_heavy<false>, dim3((unsigned)blocks), dim3(kBlock), s,
               reinterpret_cast<const f32x4*>(E), c->seg_of_row, c->offsets, c->perm, m, cols4, H, rows_per_block);
}

// ---- pseudo-targets (Algorithm 1 step 3, Eq. 6) and the pseudo-loss (Eq. 7) -------------
//
// Ht[j,:] = E[j,:] - G[row of item j,:] for the unique items of the current batch, with G the
// gradient accumulated so far in the window (this batch included), and
// loss = 1/2 sum |Ht - E|^2 = 1/2 sum G^2 over those rows.  A block takes kPseudoRows items;
// its threads add their squares in double, the block adds the thread sums in a fixed tree
// and writes one partial; k_pseudo_loss adds the partials in index order: no atomics, the
// same bits on every run.  An item whose row was dropped (buffer full) keeps Ht = E.
__global__ __launch_bounds__(kBlock) void k_pseudo_target(const f32x4* __restrict__ E,
                                                          const f32x4* __restrict__ G,
                                                          const int* __restrict__ seg_slot,
                                                          const int* __restrict__ u_ws, int cols4,
                                                          f32x4* __restrict__ Ht,
                                                          double* __restrict__ partial)
{
    __shared__ double s_sum[kBlock];
    const int U = *u_ws;
    const int j0 = blockIdx.x * kPseudoRows;
    double sum = 0.0;
    if (j0 < U) {
        const int rows = U - j0 < kPseudoRows ? U - j0 : kPseudoRows;
        const int total = rows * cols4;
        for (int e = threadIdx.x; e < total; e += kBlock) {
            const int r = e / cols4, cq = e - r * cols4;
            const int code = seg_slot[j0 + r];
            f32x4 g = {0.f, 0.f, 0.f, 0.f};
            if (code >= 0) g = G[(int64_t)(code & (kSlotNew - 1)) * cols4 + cq];
            const f32x4 h = E[(int64_t)(j0 + r) * cols4 + cq];
            if (Ht) __builtin_nontemporal_store(h - g, &Ht[(int64_t)(j0 + r) * cols4 + cq]);
            sum += (double)g.x * g.x + (double)g.y * g.y + (double)g.z * g.z + (double)g.w * g.w;
        }
    }
    s_sum[threadIdx.x] = sum;
    __syncthreads();
    for (int w = kBlock / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s_sum[threadIdx.x] += s_sum[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = s_sum[0];
}

__global__ __launch_bounds__(kBlock) void k_pseudo_loss(const double* __restrict__ partial,
                                                        const int* __restrict__ u_ws,
                                                        double* __restrict__ loss)
{
    __shared__ double s_sum[kBlock];
    const int n = (*u_ws + kPseudoRows - 1) / kPseudoRows;
    // thread t adds partials t, t + 256, ... in ascending order, then the fixed tree
    double sum = 0.0;
    for (int i = threadIdx.x; i < n; i += kBlock) sum += partial[i];
    s_sum[threadIdx.x] = sum;
    __syncthreads();
    for (int w = kBlock / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s_sum[threadIdx.x] += s_sum[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = 0.5 * s_sum[0];
}

void pseudo_target(Ctx* c, const float* E, float* Ht, double* loss_dev, hipStream_t s)
{
    const int64_t rows_max = c->cur_m < c->cap_u ? c->cur_m : c->cap_u;
    const int64_t blocks = (rows_max + kPseudoRows - 1) / kPseudoRows;
    if (blocks > 0)
        launch(c, KID_PSEUDO_TARGET, k_pseudo_target, dim3((unsigned)blocks), dim3(kBlock), s,
               reinterpret_cast<const f32x4*>(E), reinterpret_cast<const f32x4*>(c->G), c->seg_slot,
               c->scal + kSU, c->cfg.d / 4, reinterpret_cast<f32x4*>(Ht), c->loss_part);
    if (loss_dev)
        launch(c, KID_PSEUDO_LOSS, k_pseudo_loss, dim3(1), dim3(kBlock), s, c->loss_part, c->scal + kSU,
               loss_dev);
}

// ---- one content-encoder batch of the update (Alg. 1 step 4, Eq. 7) ---------
//
// The caller lists the items of the batch.  The IDs are copied once, checked: an ID outside
// [0, N) is replaced by a harmless one (the padding item, else item 0) and latches the range
// error, so the contraction kernels never form an address from it.
__global__ __launch_bounds__(kBlock) void k_chunk_ids(const int* __restrict__ ids, int n, int vocab_n,
                                                      int fix_id, int* __restrict__ out,
                                                      int* __restrict__ scal)
{
    const int j = blockIdx.x * kBlock + threadIdx.x;
    if (j == 0) scal[kSChunkN] = n;
    if (j >= n) return;
    int id = ids[j];
    if (id < 0 || id >= vocab_n) {
        id = fix_id;
        atomicOr(&scal[kSErr], kErrBitRange);
    }
    out[j] = id;
}

void chunk_ids_prepare(Ctx* c, const int* ids, int64_t n, hipStream_t s)
{
    const int64_t blocks = n > 0 ? (n + kBlock - 1) / kBlock : 1;
    launch(c, KID_CHUNK_IDS, k_chunk_ids, dim3((unsigned)blocks), dim3(kBlock), s, ids, (int)n,
           c->cfg.vocab_n, c->cfg.pad_id >= 0 ? c->cfg.pad_id : 0, c->chunk_ids, c->scal);
}

// With Ht: R[j,:] holds the encoder's output for item j of the batch and becomes the regression
// miss R[j,:] - Ht[j,:] (zero for the padding item).  Without: R already holds the miss (the
// contraction subtracted the targets as it stored).  Either way the block's share of sum |miss|^2
// goes to partial[] exactly as in k_pseudo_target (double per thread, fixed tree, k_pseudo_loss
// adds the blocks in index order).
__global__ __launch_bounds__(kBlock) void k_pseudo_miss(f32x4* __restrict__ R,
                                                        const f32x4* __restrict__ Ht,
                                                        const int* __restrict__ ids, int n, int pad_id,
                                                        int cols4, double* __restrict__ partial,
                                                        uint2* __restrict__ R_bf16)
{
    __shared__ double s_sum[kBlock];
    const int j0 = blockIdx.x * kPseudoRows;
    double sum = 0.0;
    const int rows = n - j0 < kPseudoRows ? n - j0 : kPseudoRows;
    const int total = rows * cols4;
    for (int e = threadIdx.x; e < total; e += kBlock) {
        const int r = e / cols4, cq = e - r * cols4;
        const int64_t at = (int64_t)(j0 + r) * cols4 + cq;
        f32x4 m;
        if (Ht) {
            m = f32x4{0.f, 0.f, 0.f, 0.f};
            if (ids[j0 + r] != pad_id) m = R[at] - __builtin_nontemporal_load(&Ht[at]);
            R[at] = m;
        } else {
            m = R[at];
        }
        // the copy rounded to bf16 (nearest even) that a following contraction takes as its operand
        if (R_bf16) R_bf16[at] = make_uint2(pack_bf16x2(m.x, m.y), pack_bf16x2(m.z, m.w));
        sum += (double)m.x * m.x + (double)m.y * m.y + (double)m.z * m.z + (double)m.w * m.w;
    }
    s_sum[threadIdx.x] = sum;
    __syncthreads();
    for (int w = kBlock / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s_sum[threadIdx.x] += s_sum[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = s_sum[0];
}

void pseudo_miss(Ctx* c, float* R, const float* Ht, int64_t n, double* loss_dev, hipStream_t s, void* R_bf16)
{
    if (!Ht && !loss_dev && !R_bf16) return;       // nothing to subtract, nothing to sum, nothing to round
    const int64_t blocks = (n + kPseudoRows - 1) / kPseudoRows;
    if (blocks > 0)
        launch(c, KID_PSEUDO_MISS, k_pseudo_miss, dim3((unsigned)blocks), dim3(kBlock), s,
               reinterpret_cast<f32x4*>(R), reinterpret_cast<const f32x4*>(Ht), c->chunk_ids, (int)n,
               c->cfg.pad_id, c->cfg.d / 4, c->loss_part, static_cast<uint2*>(R_bf16));
    if (loss_dev)
        launch(c, KID_PSEUDO_LOSS, k_pseudo_loss, dim3(1), dim3(kBlock), s, c->loss_part,
               c->scal + kSChunkN, loss_dev);
}

// ---- buffer rows for the items of this batch --------------------------------
//
// An item seen for the first time in the window gets the next free row of the
// persistent buffer; new items of one batch take consecutive rows in ascending
// ID order (a scan over "is new" flags), so the row layout, and with it the
// summation order of the weight gradient, is a function of the data alone.
// The dedup kernels normally work these rows out themselves (seg_slot) and the segment
// reduction commits them; the kernels below do the same job in launches of their own when the
// slot table has changed since the dedup looked at it, for an empty batch, and for the
// dense layout.

__global__ __launch_bounds__(kBlock) void k_slot_count(const int* __restrict__ uniq_ws,
                                                       const int* __restrict__ slot_of,
                                                       int* __restrict__ scal,
                                                       int* __restrict__ tile_sums, int first_step)
{
    __shared__ int sm[kWavesPerBlock];
    const int u = scal[kSU];
    const int j0 = blockIdx.x * kScanTile + threadIdx.x * 4;
    int s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (j0 + i < u) s += slot_of[uniq_ws[j0 + i]] < 0 ? 1 : 0;
    const int tot = block_sum(s, sm);
    if (threadIdx.x == 0) {
        tile_sums[blockIdx.x] = tot;
        if (blockIdx.x == 0) {
            scal[kSUBase] = first_step ? 0 : scal[kSUTotal];   // a flush leaves the old count behind
            scal[kSLongCount] = 0;
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_slot_emit(
    const int* __restrict__ uniq_ws, const int* __restrict__ offsets, int* __restrict__ slot_of,
    int* __restrict__ id_of_slot, long long* __restrict__ cnt_of_slot, int* __restrict__ seg_slot,
    int* __restrict__ scal, const int* __restrict__ tile_sums, int cap_total)
{
    __shared__ int sm[kWavesPerBlock];
    const int u = scal[kSU];
    const int u_base = scal[kSUBase];
    int pre = 0;
    for (int t = threadIdx.x; t < (int)blockIdx.x; t += kBlock) pre += tile_sums[t];
    pre = block_sum(pre, sm);

    const int j0 = blockIdx.x * kScanTile + threadIdx.x * 4;
    int id[4], old[4], s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        id[i] = 0;
        old[i] = 0;
        if (j0 + i < u) {
            id[i] = uniq_ws[j0 + i];
            old[i] = slot_of[id[i]];
            s += old[i] < 0 ? 1 : 0;
        }
    }
    int total;
    int run = u_base + pre + block_excl_scan(s, &total, sm);
    bool overflow = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int j = j0 + i;
        if (j < u) {
            const int cnt = offsets[j + 1] - offsets[j];
            if (old[i] < 0) {
                const int slot = run++;
                if (slot < cap_total) {
                    slot_of[id[i]] = slot;
                    id_of_slot[slot] = id[i];
                    cnt_of_slot[slot] = cnt;
                    seg_slot[j] = slot | kSlotNew;
                } else {
                    seg_slot[j] = -1;      // dropped: the buffer is full
                    overflow = true;
                }
            } else {
                cnt_of_slot[old[i]] += cnt;
                seg_slot[j] = old[i];
            }
        }
    }
    if (overflow) atomicOr(&scal[kSErr], kErrBitCapacity);
    // tiles past U add nothing, so the last block of the grid sees the full count
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        const int nt = u_base + pre + total;
        scal[kSUTotal] = nt < cap_total ? nt : cap_total;
    }
}

// Small batches: the same result from one block of 1024 threads that walks tiles of 4096 items in
// order (one launch, and for most small batches one pass).
constexpr int kSlotSmallThreads = 1024;
__global__ __launch_bounds__(kSlotSmallThreads) void k_slot_small(
    const int* __restrict__ uniq_ws, const int* __restrict__ offsets, int* __restrict__ slot_of,
    int* __restrict__ id_of_slot, long long* __restrict__ cnt_of_slot, int* __restrict__ seg_slot,
    int* __restrict__ scal, int cap_total, int first_step)
{
    __shared__ int sm[kSlotSmallThreads / kWave];
    const int u = scal[kSU];
    int run_base = first_step ? 0 : scal[kSUTotal];             // a flush leaves the old count behind
    bool overflow = false;
    const int t4 = (int)threadIdx.x * 4;
    for (int j0 = t4; j0 - t4 < u; j0 += kSlotSmallThreads * 4) {   // uniform trip count
        int id[4], old[4], sflag = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            id[i] = 0;
            old[i] = 0;
            if (j0 + i < u) {
                id[i] = uniq_ws[j0 + i];
                old[i] = slot_of[id[i]];
                sflag += old[i] < 0 ? 1 : 0;
            }
        }
        int total;
        int run = run_base + block_excl_scan<kSlotSmallThreads / kWave>(sflag, &total, sm);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = j0 + i;
            if (j < u) {
                const int cnt = offsets[j + 1] - offsets[j];
                if (old[i] < 0) {
                    const int slot = run++;
                    if (slot < cap_total) {
                        slot_of[id[i]] = slot;
                        id_of_slot[slot] = id[i];
                        cnt_of_slot[slot] = cnt;
                        seg_slot[j] = slot | kSlotNew;
                    } else {
                        seg_slot[j] = -1;
                        overflow = true;
                    }
                } else {
                    cnt_of_slot[old[i]] += cnt;
                    seg_slot[j] = old[i];
                }
            }
        }
        run_base += total;
    }
    if (overflow) atomicOr(&scal[kSErr], kErrBitCapacity);
    __syncthreads();      // every thread has read scal[kSUTotal] before it changes
    if (threadIdx.x == 0) {
        scal[kSUTotal] = run_base < cap_total ? run_base : cap_total;
        scal[kSLongCount] = 0;
    }
}

constexpr int64_t kSmallBatch = 8 * kScanTile;   // positions up to which one-block variants are used

// Dense-by-vocabulary buffer: the row of an item is its ID, so there is nothing to hand out; the
// row is always added to (rows outside a window are zero) and the 64-bit count of the item grows.
__global__ __launch_bounds__(kBlock) void k_slot_dense(const int* __restrict__ uniq_ws,
                                                       const int* __restrict__ offsets,
                                                       int* __restrict__ scal,
                                                       long long* __restrict__ cnt64,
                                                       int* __restrict__ seg_slot, int vocab_n)
{
    const int j = blockIdx.x * kBlock + threadIdx.x;
    if (j == 0) {
        scal[kSLongCount] = 0;
        scal[kSUTotal] = vocab_n;      // rows the weight gradient contracts over: all of them
    }
    if (j >= scal[kSU]) return;
    const int id = uniq_ws[j];         // distinct within a batch: no two threads meet on a count
    seg_slot[j] = id;
    cnt64[id] += offsets[j + 1] - offsets[j];
}

void assign_slots(Ctx* c, hipStream_t s)
{
    int64_t bound = c->cur_m < c->cap_u ? c->cur_m : c->cap_u;
    if (bound < 1) bound = 1;
    if (c->dense) {
        launch(c, KID_SLOT_EMIT, k_slot_dense, dim3((unsigned)((bound + kBlock - 1) / kBlock)), dim3(kBlock), s,
               c->uniq_ws, c->offsets, c->scal, c->cnt64, c->seg_slot, c->cfg.vocab_n);
        return;
    }
    const int first_step = (c->steps_done == 0 && !c->window_imported) ? 1 : 0;
    if (bound <= kSmallBatch) {
        launch(c, KID_SLOT_EMIT, k_slot_small, dim3(1), dim3(kSlotSmallThreads), s, c->uniq_ws, c->offsets, c->slot_of,
               c->id_of_slot, c->cnt_of_slot, c->seg_slot, c->scal, (int)c->cap_total, first_step);
        return;
    }
    const int tiles = (int)((bound + kScanTile - 1) / kScanTile);
    launch(c, KID_SLOT_COUNT, k_slot_count, dim3(tiles), dim3(kBlock), s, c->uniq_ws, c->slot_of, c->scal,
                       c->tile_sums, first_step);
    launch(c, KID_SLOT_EMIT, k_slot_emit, dim3(tiles), dim3(kBlock), s, c->uniq_ws, c->offsets,
                       c->slot_of, c->id_of_slot, c->cnt_of_slot, c->seg_slot, c->scal, c->tile_sums,
                       (int)c->cap_total);
}

// ---- sorted-segment reduction -----------------------------------------------
//
// Rows of dH are visited in the sorted order of the batch (perm), where the
// occurrences of one item are adjacent and in ascending position.  The sorted
// rows are cut into tiles of kSegRows.
//  * A short segment (< seg_long rows: kSegLong, or kSegLongSmall for small batches) is summed, whole and in order, by the
//    tile that holds its first row, even where it runs past the tile's end; it
//    needs no partial result.
//  * A long segment is summed tile by tile into partial rows (seg_last for the
//    tile where it starts, seg_first for every later tile), and k_seg_combine
//    adds the partials in ascending tile order.
// Destination codes kept per row in LDS:
constexpr int kDstNone = -1;    // nothing to write (dropped item)
constexpr int kDstFirst = -2;   // partial row seg_first[tile]
constexpr int kDstLast = -3;    // partial row seg_last[tile]
constexpr int kSegMaxRows = kSegRows + kSegLong;
constexpr int kSegUnroll = 16;
constexpr int kSegPlainLoads = 16384;   // batches of at most this many positions read dH with plain loads

__device__ __forceinline__ void write_final(float4* __restrict__ G, int cols4, int col, int code,
                                            bool is_pad, float4 acc)
{
    if (code == kDstNone) return;
    float4* dst = G + (int64_t)(code & (kSlotNew - 1)) * cols4 + col;
    if (code & kSlotNew) {
        // a row new to the window is not read again before the next step at the earliest: stored past
        // the caches, it leaves them to the forward's operands (measured: 8 us per step on the large shape)
        const float4 w = is_pad ? make_float4(0.f, 0.f, 0.f, 0.f) : acc;
        __builtin_nontemporal_store(f32x4{w.x, w.y, w.z, w.w}, reinterpret_cast<f32x4*>(dst));
    } else if (!is_pad) {
        *dst = f4_add(*dst, acc);
    }
}

template <bool PLAIN>      // dH read with plain instead of non-temporal loads
__global__ __launch_bounds__(kBlock) void k_seg_reduce(
    const float4* __restrict__ dH, const int* __restrict__ perm, const int* __restrict__ seg_of_row,
    const int* __restrict__ offsets, const int* __restrict__ uniq_ws,
    const int* __restrict__ seg_slot, int n, int cols4, int pad_id, float4* __restrict__ G,
    float4* __restrict__ seg_first, float4* __restrict__ seg_last, int* __restrict__ scal,
    int* __restrict__ long_list, int seg_long, int* __restrict__ slot_of, int* __restrict__ id_of_slot,
    long long* __restrict__ cnt_of_slot)
{
    __shared__ __attribute__((aligned(16))) int s_src[kSegMaxRows];    // dH row of each sorted row, -1 = padding (not read)
    __shared__ __attribute__((aligned(16))) int s_dst[kSegMaxRows];    // 0 = keep adding; else destination code + 4 (see below)
    static_assert(kSegMaxRows % kSegUnroll == 0, "a group of rows is read from the tables as whole 16-byte pieces");
    __shared__ int s_pad[kSegMaxRows];

    const int t = blockIdx.x;
    const int r0 = t * kSegRows;
    const int r1 = r0 + kSegRows < n ? r0 + kSegRows : n;
    // slot_of given: the buffer rows in seg_slot were worked out by the dedup and are committed
    // here, each item by the thread that meets the first row of its segment (one tile holds it)
    const bool commit = slot_of != nullptr && blockIdx.y == 0;
    if (commit && t == 0 && threadIdx.x == 0) scal[kSUTotal] = scal[kSUNext];

    // first and one-past-last sorted row this tile sums
    int a, b;
    {
        const int sg = seg_of_row[r0];
        const int o0 = offsets[sg], o1 = offsets[sg + 1];
        a = (o0 < r0 && o1 - o0 < seg_long) ? o1 : r0;
        const int sl = seg_of_row[r1 - 1];
        const int p0 = offsets[sl], p1 = offsets[sl + 1];
        b = (p1 - p0 < seg_long) ? p1 : r1;
    }
    if (a >= r1) return;      // the tile lies inside a short segment owned by an earlier tile
    const int rows = b - a;

    for (int i = threadIdx.x; i < rows; i += blockDim.x) {
        const int r = a + i;
        const int sg = seg_of_row[r];
        const int o0 = offsets[sg], o1 = offsets[sg + 1];
        const bool is_long = o1 - o0 >= seg_long;
        const bool is_pad = uniq_ws[sg] == pad_id;
        const bool seg_end = r + 1 == o1;
        int code = 0;
        if (is_long) {
            if (seg_end || r + 1 == r1) code = (o0 < r0 ? kDstFirst : kDstLast) + 4;
        } else if (seg_end) {
            code = seg_slot[sg] + 4;
        }
        s_src[i] = is_pad ? -1 : perm[r];
        s_dst[i] = code;
        s_pad[i] = is_pad ? 1 : 0;
        if (commit && r == o0) {
            const int row = seg_slot[sg];
            if (row < 0) {
                atomicOr(&scal[kSErr], kErrBitCapacity);      // dropped: the buffer is full
            } else if (row & kSlotNew) {
                const int id = uniq_ws[sg], slot = row & (kSlotNew - 1);
                slot_of[id] = slot;
                id_of_slot[slot] = id;
                cnt_of_slot[slot] = o1 - o0;
            } else {
                cnt_of_slot[row] += o1 - o0;
            }
        }
    }
    __syncthreads();

    const int col = blockIdx.y * blockDim.x + threadIdx.x;
    if (col >= cols4) return;

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i0 = 0; i0 < rows; i0 += kSegUnroll) {
        float4 v[kSegUnroll];
        // the group's table entries first, as 16-byte LDS reads: fetched one by one, each row's load
        // would be issued an LDS round trip after the one before it
        int srcs[kSegUnroll], codes[kSegUnroll];
#pragma unroll
        for (int q = 0; q < kSegUnroll / 4; ++q) {
            const int4 a = *reinterpret_cast<const int4*>(&s_src[i0 + 4 * q]);
            const int4 b = *reinterpret_cast<const int4*>(&s_dst[i0 + 4 * q]);
            srcs[4 * q] = a.x; srcs[4 * q + 1] = a.y; srcs[4 * q + 2] = a.z; srcs[4 * q + 3] = a.w;
            codes[4 * q] = b.x; codes[4 * q + 1] = b.y; codes[4 * q + 2] = b.z; codes[4 * q + 3] = b.w;
        }
#pragma unroll
        for (int k = 0; k < kSegUnroll; ++k) {
            const int i = i0 + k;
            const int src = i < rows ? srcs[k] : -1;
            // every row of dH is read exactly once: stream it past the caches (batches of a few
            // thousand positions are better off with plain loads: their rows often still sit in a
            // cache, and what they have to hide is latency; measured 1 to 1.4 us per step).  The
            // choice is made at compile time: chosen at run time inside this loop it cost the large
            // shape 10 % of the kernel
            v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (src >= 0) {
                const f32x4* p = reinterpret_cast<const f32x4*>(dH) + (int64_t)src * cols4 + col;
                const f32x4 t = PLAIN ? *p : __builtin_nontemporal_load(p);
                v[k] = make_float4(t.x, t.y, t.z, t.w);
            }
        }
#pragma unroll
        for (int k = 0; k < kSegUnroll; ++k) {
            const int i = i0 + k;
            if (i < rows) {
                acc = f4_add(acc, v[k]);
                const int code = codes[k];
                if (code != 0) {
                    const int dst = code - 4;
                    if (dst == kDstFirst) {
                        seg_first[(int64_t)t * cols4 + col] = acc;
                    } else if (dst == kDstLast) {
                        seg_last[(int64_t)t * cols4 + col] = acc;
                        if (col == 0) long_list[atomicAdd(&scal[kSLongCount], 1)] = t;
                    } else {
                        write_final(G, cols4, col, dst, s_pad[i] != 0, acc);
                    }
                    acc = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        }
    }
}

// Sum of a long segment's partial rows in ascending tile order.  A block owns
// kFixCols4 float4 columns; its kFixLanes row lanes each add every
// kFixLanes-th partial, then lane sums are added in lane order.
__global__ __launch_bounds__(kBlock) void k_seg_combine(
    const int* __restrict__ seg_of_row, const int* __restrict__ offsets,
    const int* __restrict__ uniq_ws, const int* __restrict__ seg_slot, int n, int cols4, int pad_id,
    float4* __restrict__ G, const float4* __restrict__ seg_first,
    const float4* __restrict__ seg_last, const int* __restrict__ scal,
    const int* __restrict__ long_list)
{
    __shared__ float4 sm[kFixLanes][kFixCols4];
    const int cl = threadIdx.x % kFixCols4;
    const int rl = threadIdx.x / kFixCols4;
    const int col = blockIdx.y * kFixCols4 + cl;
    const int count = scal[kSLongCount];
    for (int w = blockIdx.x; w < count; w += gridDim.x) {
        const int t = long_list[w];
        int last_row = (t + 1) * kSegRows - 1;
        if (last_row > n - 1) last_row = n - 1;
        const int sg = seg_of_row[last_row];
        const int seg_end = offsets[sg + 1];
        const bool is_pad = uniq_ws[sg] == pad_id;
        // partial i: i = 0 -> seg_last[t]; i >= 1 -> seg_first[t + i]
        const int parts = 1 + (seg_end - 1) / kSegRows - t;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!is_pad && col < cols4) {
            // the lane's partials are fetched eight at a time (the adds keep their order): one
            // load per round trip would make the longest segment's chain the kernel's duration
            constexpr int kAhead = 8;
            for (int i0 = rl; i0 < parts; i0 += kFixLanes * kAhead) {
                float4 v[kAhead];
#pragma unroll
                for (int k = 0; k < kAhead; ++k) {
                    const int i = i0 + k * kFixLanes;
                    const float4* src = i == 0 ? seg_last + (int64_t)t * cols4
                                               : seg_first + (int64_t)(t + i) * cols4;
                    v[k] = i < parts ? src[col] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int k = 0; k < kAhead; ++k)
                    if (i0 + k * kFixLanes < parts) acc = f4_add(acc, v[k]);
            }
        }
        sm[rl][cl] = acc;
        __syncthreads();
        if (rl == 0 && col < cols4) {
            float4 tot = sm[0][cl];
#pragma unroll
            for (int k = 1; k < kFixLanes; ++k) tot = f4_add(tot, sm[k][cl]);
            write_final(G, cols4, col, seg_slot[sg], is_pad, tot);
        }
        __syncthreads();
    }
}

// commit: seg_slot holds rows worked out by the dedup; the reduction writes them into the slot table
void segment_reduce(Ctx* c, const float* dH, int64_t m, hipStream_t s, bool commit)
{
    if (m == 0) return;
    const int n = (int)m;
    const int cols4 = c->cfg.d / 4;
    int threads = ((cols4 + kWave - 1) / kWave) * kWave;
    if (threads > kBlock) threads = kBlock;
    const int slabs = (cols4 + threads - 1) / threads;
    // Whole-segment sums are one block's serial chain of row loads: short chains matter most when
    // the batch has few tiles to hide them behind.
    const int seg_long = n > kSegSmallBatch ? kSegLong : kSegLongSmall;
    const int tiles = (n + kSegRows - 1) / kSegRows;
    if (n > kSegPlainLoads)
        launch(c, KID_SEG_REDUCE, k_seg_reduce<false>, dim3(tiles, slabs), dim3(threads), s,
                           reinterpret_cast<const float4*>(dH), c->perm, c->seg_of_row, c->offsets,
                           c->uniq_ws, c->seg_slot, n, cols4, c->cfg.pad_id,
                           reinterpret_cast<float4*>(c->G), reinterpret_cast<float4*>(c->seg_first),
                           reinterpret_cast<float4*>(c->seg_last), c->scal, c->long_list, seg_long,
                           commit ? c->slot_of : (int*)nullptr, c->id_of_slot, c->cnt_of_slot);
    else
        launch(c, KID_SEG_REDUCE, k_seg_reduce<true>, dim3(tiles, slabs), dim3(threads), s,
                           reinterpret_cast<const float4*>(dH), c->perm, c->seg_of_row, c->offsets,
                           c->uniq_ws, c->seg_slot, n, cols4, c->cfg.pad_id,
                           reinterpret_cast<float4*>(c->G), reinterpret_cast<float4*>(c->seg_first),
                           reinterpret_cast<float4*>(c->seg_last), c->scal, c->long_list, seg_long,
                           commit ? c->slot_of : (int*)nullptr, c->id_of_slot, c->cnt_of_slot);
    int fix_blocks = tiles / (seg_long / kSegRows) + 1;   // upper bound of long segments
    if (fix_blocks > 1024) fix_blocks = 1024;        // a block per long segment for all but extreme batches
    launch(c, KID_SEG_COMBINE, k_seg_combine, dim3(fix_blocks, (cols4 + kFixCols4 - 1) / kFixCols4),
                       dim3(kBlock), s, c->seg_of_row, c->offsets, c->uniq_ws, c->seg_slot, n,
                       cols4, c->cfg.pad_id, reinterpret_cast<float4*>(c->G),
                       reinterpret_cast<const float4*>(c->seg_first),
                       reinterpret_cast<const float4*>(c->seg_last), c->scal, c->long_list);
}

// ---- end of the window: export in ascending ID order, then empty ------------
//
// One launch: rows of G are copied out in ascending ID order while a few extra blocks export the
// IDs and counts and clear the items' entries of the slot map.
// The count of buffer rows (scal[kSUTotal]) is left as it is: every block reads it here, and
// the first step of the next window starts from zero by itself.  `n_zero`: the window is empty.

// rank_of_slot (nullable, needs sorted_slots): receives, for every buffer row, its place in
// ascending-ID order, for a weight-gradient kernel that writes the rows out itself.
__global__ __launch_bounds__(kBlock) void k_flush_meta(
    const int* __restrict__ sorted_ids, const int* __restrict__ sorted_slots,
    const long long* __restrict__ cnt_of_slot, int* __restrict__ slot_of, int* __restrict__ uniq_total,
    int* __restrict__ counts_total, long long* __restrict__ counts64_total, int* __restrict__ scal,
    int* __restrict__ u_total_dev, int n_zero, int* __restrict__ rank_of_slot)
{
    const int n = n_zero ? 0 : scal[kSUTotal];
    for (int r = blockIdx.x * kBlock + threadIdx.x; r < n; r += gridDim.x * kBlock) {
        flush_meta_row(r, sorted_ids, sorted_slots, cnt_of_slot, slot_of, uniq_total, counts_total,
                       counts64_total);
        if (rank_of_slot) rank_of_slot[sorted_slots[r]] = r;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (u_total_dev) *u_total_dev = n;
        scal[kSFlushN] = n;
    }
}

// Blocks [0, copy_blocks) copy rows; the blocks after them export IDs and counts and clear the
// slot map (kept out of the copy loop: their scattered accesses would stall the copying waves).
__global__ __launch_bounds__(kBlock) void k_flush_rows(
    const int* __restrict__ sorted_ids, const int* __restrict__ sorted_slots,
    const long long* __restrict__ cnt_of_slot, int* __restrict__ slot_of, int* __restrict__ uniq_total,
    int* __restrict__ counts_total, long long* __restrict__ counts64_total,
    const float4* __restrict__ G, int cols4, float4* __restrict__ G_total, int* __restrict__ scal,
    int* __restrict__ u_total_dev, int copy_blocks)
{
    const int n = scal[kSUTotal];
    if ((int)blockIdx.x >= copy_blocks) {
        const int mb = blockIdx.x - copy_blocks, nmb = gridDim.x - copy_blocks;
        for (int r = mb * kBlock + threadIdx.x; r < n; r += nmb * kBlock)
            flush_meta_row(r, sorted_ids, sorted_slots, cnt_of_slot, slot_of, uniq_total, counts_total,
                           counts64_total);
        if (mb == 0 && threadIdx.x == 0) {
            if (u_total_dev) *u_total_dev = n;
            scal[kSFlushN] = n;
        }
        return;
    }
    const int64_t total = (int64_t)n * cols4;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
         i += (int64_t)copy_blocks * kBlock) {
        const int64_t r = i / cols4;
        const int cc = (int)(i % cols4);
        const f32x4 t = __builtin_nontemporal_load(
            reinterpret_cast<const f32x4*>(G) + (int64_t)(sorted_slots ? sorted_slots[r] : (int)r) * cols4 + cc);
        __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(G_total) + i);
    }
}

void flush_export(Ctx* c, int* uniq_total, int* counts_total, long long* counts64_total, float* G_total,
                  int* u_total_dev, hipStream_t s)
{
    if (c->steps_done == 0 && !c->window_imported) {       // nothing accumulated since the last flush
        launch(c, KID_FLUSH_META, k_flush_meta, dim3(1), dim3(kBlock), s, c->id_of_slot, (const int*)nullptr,
               c->cnt_of_slot, c->slot_of, uniq_total, counts_total, counts64_total, c->scal, u_total_dev, 1,
               (int*)nullptr);
        return;
    }
    // After one step the buffer rows are already in ascending ID order (rows are handed out in
    // that order within a step); only later steps append out of order.
    const int* sorted_ids = c->id_of_slot;
    const int* sorted_slots = nullptr;
    if (c->steps_done > 1 || c->window_imported) {
        const int r = radix_sort_pairs(c, c->id_of_slot, nullptr, 0, c->scal + kSUTotal, c->cap_total,
                                       false, 0, s);
        sorted_ids = c->keys[r];
        sorted_slots = c->vals[r];
    }
    if (G_total) {
        int64_t blocks = (c->cap_total * (c->cfg.d / 4) + kBlock - 1) / kBlock;
        if (blocks > 2048) blocks = 2048;
        int64_t meta_blocks = (c->cap_total + kBlock - 1) / kBlock;
        if (meta_blocks > 64) meta_blocks = 64;
        launch(c, KID_FLUSH_ROWS, k_flush_rows, dim3((unsigned)(blocks + meta_blocks)), dim3(kBlock), s, sorted_ids,
               sorted_slots, c->cnt_of_slot, c->slot_of, uniq_total, counts_total, counts64_total,
               reinterpret_cast<const float4*>(c->G), c->cfg.d / 4, reinterpret_cast<float4*>(G_total), c->scal,
               u_total_dev, (int)blocks);
    } else {
        int64_t blocks = (c->cap_total + kBlock - 1) / kBlock;
        if (blocks > 1024) blocks = 1024;
        launch(c, KID_FLUSH_META, k_flush_meta, dim3((unsigned)blocks), dim3(kBlock), s, sorted_ids,
               sorted_slots, c->cnt_of_slot, c->slot_of, uniq_total, counts_total, counts64_total, c->scal,
               u_total_dev, 0, (int*)nullptr);
    }
}

// The export without the rows: IDs and counts in ascending-ID order, slot map cleared, and the
// place of every buffer row in that order (returned; NULL: the rows are in that order already).
// The caller's weight-gradient kernel then writes the rows themselves.  Needs a non-empty window.
// *left_to_caller: nothing was launched (a one-step window); the caller's kernel does this part too.
const int* flush_meta_and_ranks(Ctx* c, int* uniq_total, int* counts_total, int* u_total_dev, hipStream_t s,
                                bool* left_to_caller)
{
    const int* sorted_ids = c->id_of_slot;
    const int* sorted_slots = nullptr;
    int* ranks = nullptr;
    *left_to_caller = false;
    if (c->steps_done <= 1 && !c->window_imported) {
        // one step: the rows are in order already and nothing has to be ranked; a few extra blocks
        // of the caller's weight-gradient launch export the IDs and counts
        *left_to_caller = true;
        return nullptr;
    }
    {
        const int r = radix_sort_pairs(c, c->id_of_slot, nullptr, 0, c->scal + kSUTotal, c->cap_total,
                                       false, 0, s);
        sorted_ids = c->keys[r];
        sorted_slots = c->vals[r];
        ranks = c->chunk_ids;          // [cap_chunk >= cap_total]: free between content-encoder batches
    }
    int64_t blocks = (c->cap_total + kBlock - 1) / kBlock;
    if (blocks > 1024) blocks = 1024;
    launch(c, KID_FLUSH_META, k_flush_meta, dim3((unsigned)blocks), dim3(kBlock), s, sorted_ids, sorted_slots,
           c->cnt_of_slot, c->slot_of, uniq_total, counts_total, (long long*)nullptr, c->scal, u_total_dev, 0,
           ranks);
    return ranks;
}

// ---- slot table: a saved window state merged into the buffer ----------------------------
//
// One block walks the listed items in tiles of 4096 exactly as k_slot_small walks the items of a
// batch: an item the window has not met takes the next free row (in list order), an item it has
// met keeps its row; the saved count is added (64-bit counts, as in the dense layout).
// code[j] receives the row (kSlotNew set for a fresh row, -1 when the buffer is full or the ID is
// outside [0, N)); k_import_rows then writes or adds the saved gradient rows.
__global__ __launch_bounds__(kSlotSmallThreads) void k_slot_import(
    const int* __restrict__ ids, const long long* __restrict__ counts, int n, int vocab_n,
    int* __restrict__ slot_of, int* __restrict__ id_of_slot, long long* __restrict__ cnt_of_slot,
    int* __restrict__ code, int* __restrict__ scal, int cap_total, int first_touch)
{
    __shared__ int sm[kSlotSmallThreads / kWave];
    int run_base = first_touch ? 0 : scal[kSUTotal];
    int err = 0;
    const int t4 = (int)threadIdx.x * 4;
    for (int j0 = t4; j0 - t4 < n; j0 += kSlotSmallThreads * 4) {   // uniform trip count
        int id[4], old[4], sflag = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            id[i] = -1;
            old[i] = 0;
            if (j0 + i < n) {
                const int v = ids[j0 + i];
                if (v >= 0 && v < vocab_n) {
                    id[i] = v;
                    old[i] = slot_of[v];
                    sflag += old[i] < 0 ? 1 : 0;
                } else {
                    err |= kErrBitRange;
                }
            }
        }
        int total;
        int run = run_base + block_excl_scan<kSlotSmallThreads / kWave>(sflag, &total, sm);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = j0 + i;
            if (j >= n) continue;
            if (id[i] < 0) {
                code[j] = -1;
                continue;
            }
            const long long c64 = counts[j];
            if (old[i] < 0) {
                const int slot = run++;
                if (slot < cap_total) {
                    slot_of[id[i]] = slot;
                    id_of_slot[slot] = id[i];
                    cnt_of_slot[slot] = c64;
                    code[j] = slot | kSlotNew;
                } else {
                    code[j] = -1;
                    err |= kErrBitCapacity;
                }
            } else {
                cnt_of_slot[old[i]] += c64;
                code[j] = old[i];
            }
        }
        run_base += total;
    }
    if (err) atomicOr(&scal[kSErr], err);
    if (threadIdx.x == 0) scal[kSUTotal] = run_base < cap_total ? run_base : cap_total;
}

__global__ __launch_bounds__(kBlock) void k_import_rows(const int* __restrict__ code,
                                                        const f32x4* __restrict__ rows, int n,
                                                        int cols4, f32x4* __restrict__ G)
{
    const int64_t total = (int64_t)n * cols4;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kBlock) {
        const int64_t r = i / cols4;
        const int cc = (int)(i % cols4);
        const int cd = code[r];
        if (cd < 0) continue;
        f32x4* dst = G + (int64_t)(cd & (kSlotNew - 1)) * cols4 + cc;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (rows) v = rows[i];
        *dst = (cd & kSlotNew) ? v : *dst + v;
    }
}

void import_slots(Ctx* c, const int* ids, const long long* counts, const float* rows, int64_t n,
                  hipStream_t s)
{
    const int first_touch = (c->steps_done == 0 && !c->window_imported) ? 1 : 0;
    launch(c, KID_SLOT_EMIT, k_slot_import, dim3(1), dim3(kSlotSmallThreads), s, ids, counts, (int)n,
           c->cfg.vocab_n, c->slot_of, c->id_of_slot, c->cnt_of_slot, c->chunk_ids, c->scal,
           (int)c->cap_total, first_touch);
    if (n == 0) return;
    int64_t blocks = (n * (c->cfg.d / 4) + kBlock - 1) / kBlock;
    if (blocks > 2048) blocks = 2048;
    launch(c, KID_FLUSH_ROWS, k_import_rows, dim3((unsigned)blocks), dim3(kBlock), s, c->chunk_ids,
           reinterpret_cast<const f32x4*>(rows), (int)n, c->cfg.d / 4, reinterpret_cast<f32x4*>(c->G));
}

// ---- dense-by-vocabulary buffer: end of the window, and resuming one --------------------
//
// The items of the window are those with a non-zero count.  Tiles of kScanTile IDs are counted,
// then every tile finds its place from the counts of the tiles before it and writes its items'
// IDs (ascending by construction) and counts, clearing the counts; a third kernel copies the
// items' rows out and zeroes them, which is what makes "always add" correct in the next window.

__global__ __launch_bounds__(kBlock) void k_dense_count(const long long* __restrict__ cnt64,
                                                        int vocab_n, int* __restrict__ tile_sums)
{
    __shared__ int sm[kWavesPerBlock];
    const int i0 = blockIdx.x * kScanTile + threadIdx.x * 4;
    int s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (i0 + i < vocab_n) s += cnt64[i0 + i] != 0 ? 1 : 0;
    const int tot = block_sum(s, sm);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = tot;
}

__global__ __launch_bounds__(kBlock) void k_dense_emit(
    long long* __restrict__ cnt64, int vocab_n, const int* __restrict__ tile_sums,
    int* __restrict__ list, int* __restrict__ uniq_total, int* __restrict__ counts_total,
    long long* __restrict__ counts64_total, int* __restrict__ scal, int* __restrict__ u_total_dev)
{
    __shared__ int sm[kWavesPerBlock];
    int pre = 0;
    for (int t = threadIdx.x; t < (int)blockIdx.x; t += kBlock) pre += tile_sums[t];
    pre = block_sum(pre, sm);
    const int i0 = blockIdx.x * kScanTile + threadIdx.x * 4;
    long long cnt[4];
    int s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        cnt[i] = i0 + i < vocab_n ? cnt64[i0 + i] : 0;
        s += cnt[i] != 0 ? 1 : 0;
    }
    int total;
    int at = pre + block_excl_scan(s, &total, sm);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (cnt[i] != 0) {
            list[at] = i0 + i;
            if (uniq_total) uniq_total[at] = i0 + i;
            if (counts_total) counts_total[at] = cnt[i] > 0x7fffffffLL ? 0x7fffffff : (int)cnt[i];
            if (counts64_total) counts64_total[at] = cnt[i];
            cnt64[i0 + i] = 0;
            ++at;
        }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        if (u_total_dev) *u_total_dev = pre + total;
        scal[kSFlushN] = pre + total;
    }
}

__global__ __launch_bounds__(kBlock) void k_dense_rows(const int* __restrict__ list,
                                                       const int* __restrict__ scal,
                                                       f32x4* __restrict__ G, int cols4,
                                                       f32x4* __restrict__ G_total)
{
    const int64_t total = (int64_t)scal[kSFlushN] * cols4;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kBlock) {
        const int64_t r = i / cols4;
        const int cc = (int)(i % cols4);
        f32x4* src = G + (int64_t)list[r] * cols4 + cc;
        if (G_total) __builtin_nontemporal_store(*src, G_total + i);
        *src = zero;
    }
}

void flush_dense(Ctx* c, int* uniq_total, int* counts_total, long long* counts64_total, float* G_total,
                 int* u_total_dev, hipStream_t s)
{
    const int n = c->cfg.vocab_n;
    const int tiles = (n + kScanTile - 1) / kScanTile;
    int* list = c->keys[0];
    launch(c, KID_FLUSH_META, k_dense_count, dim3(tiles), dim3(kBlock), s, c->cnt64, n, c->dense_sums);
    launch(c, KID_FLUSH_META, k_dense_emit, dim3(tiles), dim3(kBlock), s, c->cnt64, n, c->dense_sums, list,
           uniq_total, counts_total, counts64_total, c->scal, u_total_dev);
    int64_t blocks = ((int64_t)n * (c->cfg.d / 4) + kBlock - 1) / kBlock;
    if (blocks > 2048) blocks = 2048;
    launch(c, KID_FLUSH_ROWS, k_dense_rows, dim3((unsigned)blocks), dim3(kBlock), s, list, c->scal,
           reinterpret_cast<f32x4*>(c->G), c->cfg.d / 4, reinterpret_cast<f32x4*>(G_total));
}

// A saved window state merged into the buffer: counts and rows of the listed (distinct) items are
// added.  An ID outside [0, N) latches the range error and is skipped.
__global__ __launch_bounds__(kBlock) void k_dense_import(const int* __restrict__ ids,
                                                         const long long* __restrict__ counts,
                                                         const f32x4* __restrict__ rows, int n,
                                                         int vocab_n, int cols4,
                                                         long long* __restrict__ cnt64,
                                                         f32x4* __restrict__ G, int* __restrict__ scal)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) scal[kSUTotal] = vocab_n;
    const int64_t total = (int64_t)n * cols4;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kBlock) {
        const int64_t r = i / cols4;
        const int cc = (int)(i % cols4);
        const int id = ids[r];
        if (id < 0 || id >= vocab_n) {
            if (cc == 0) atomicOr(&scal[kSErr], kErrBitRange);
            continue;
        }
        if (cc == 0) cnt64[id] += counts[r];
        if (rows) {
            f32x4* dst = G + (int64_t)id * cols4 + cc;
            *dst = *dst + rows[i];
        }
    }
}

void import_dense(Ctx* c, const int* ids, const long long* counts, const float* rows, int64_t n,
                  hipStream_t s)
{
    int64_t blocks = (n * (c->cfg.d / 4) + kBlock - 1) / kBlock;
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    launch(c, KID_FLUSH_ROWS, k_dense_import, dim3((unsigned)blocks), dim3(kBlock), s, ids, counts,
           reinterpret_cast<const f32x4*>(rows), (int)n, c->cfg.vocab_n, c->cfg.d / 4, c->cnt64,
           reinterpret_cast<f32x4*>(c->G), c->scal);
}

}  // namespace gram
