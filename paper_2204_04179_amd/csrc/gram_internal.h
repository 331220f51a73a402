// Internal declarations shared by the translation units of libgram (HIP, gfx950).
// Not part of the public ABI; see include/gram.h for that.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include <string>
#include <utility>
#include <vector>

#include "gram.h"

namespace gram {

constexpr int kWave = 64;
constexpr int kBlock = 256;             // threads of the integer / streaming kernels
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kMaxDigitBits = 10;       // radix digit width limit (1024 LDS bins per wave)
constexpr int kScanTile = 1024;         // rows per block in the flag-scan kernels
constexpr int kSegRows = 32;            // sorted rows per tile of the segment reduction
constexpr int kSegLong = 64;            // segments with at least this many rows are reduced tile by tile ...
constexpr int kSegLongSmall = 32;       // ... or this many when the batch has at most kSegSmallBatch positions
constexpr int kSegSmallBatch = 65536;
constexpr int kLightMax = 32;           // items with more positions are gathered by a separate copy kernel
constexpr int kSlotNew = 1 << 30;       // flag in seg_slot: the buffer row is created by this step
constexpr int kPseudoRows = 8;          // unique items per block of the pseudo-target kernel
constexpr int kFixCols4 = 16;           // float4 columns per block of the long-segment combine
constexpr int kFixLanes = kBlock / kFixCols4;
// A buffer descriptor addresses base + 32-bit byte offset: matrices of at least this many bytes
// take the kernels' wide-address variants.
constexpr int64_t kBufferWindow = ((int64_t)1 << 32) - 16;

// Export of one item at the end of a window: ID and count of the r-th item in ascending-ID order
// (sorted_slots NULL: buffer row r), its entry of the slot map cleared.
__device__ __forceinline__ void flush_meta_row(int r, const int* sorted_ids, const int* sorted_slots,
                                               const long long* cnt_of_slot, int* slot_of, int* uniq_total,
                                               int* counts_total, long long* counts64_total)
{
    const int id = sorted_ids[r];
    const long long cnt = cnt_of_slot[sorted_slots ? sorted_slots[r] : r];
    if (uniq_total) uniq_total[r] = id;
    if (counts_total) counts_total[r] = cnt > 0x7fffffffLL ? 0x7fffffff : (int)cnt;     // the 32-bit export saturates
    if (counts64_total) counts64_total[r] = cnt;
    slot_of[id] = -1;
}

// two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef float f32x2_ __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_ __attribute__((ext_vector_type(2)));
    const f32x2_ v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_));
}

// Device scalars (ctx->scal[...]).
enum Scalar { kSU = 0, kSUTotal, kSErr, kSUBase, kSLongCount, kSFlushN, kSChunkN, kSUNext, kSCount };

// Device-latched error bits (scal[kSErr]).
constexpr int kErrBitRange = 1;
constexpr int kErrBitCapacity = 2;

// Kernel identifiers for the built-in event timer (gram_profile_*).
enum KernelId {
    KID_RADIX_HIST = 0, KID_RADIX_SCAN, KID_RADIX_SCATTER, KID_HEADS_COUNT, KID_HEADS_EMIT,
    KID_UNIQUE_EMPTY, KID_TRANSPOSE_U16, KID_ENCODE_BF16, KID_ENCODE_F32, KID_GATHER_ROWS,
    KID_SLOT_COUNT, KID_SLOT_EMIT, KID_SEG_REDUCE, KID_SEG_COMBINE, KID_WGRAD_BF16, KID_WGRAD_F32,
    KID_WGRAD_REDUCE, KID_FLUSH_META, KID_FLUSH_ROWS, KID_UNIQUE_SMALL,
    KID_GATHER_HEAVY, KID_PSEUDO_TARGET, KID_PSEUDO_LOSS, KID_CHUNK_IDS, KID_PSEUDO_MISS, KID_MLP_TO_BF16,
    KID_ENCODE_BF16_WIDE, KID_WGRAD_BF16_WIDE, KID_COUNT
};

static_assert(KID_COUNT <= 64, "the profiling mask has 64 bits");

struct ProfSlot {
    hipEvent_t start, stop;
    int kid;
};

struct SortPlan {
    int passes;
    int digit_bits[4];
    int items;   // 64-key rounds per wave
    int nw;      // waves (chunks) over the host upper bound of n
    int blocks;
};

struct Ctx {
    gram_config cfg;
    int64_t cap_u;        // min(max_positions, vocab_n): upper bound of U per step
    int64_t cap_total;    // rows of the persistent buffer
    bool dense = false;   // buffer_layout == GRAM_BUFFER_DENSE: row of an item = its ID, no slot map
    int64_t cap_chunk;    // max(cap_u, cap_total): upper bound of a content-encoder batch
    int key_bits;         // bits needed for an ID

    // --- workspace (device) ---
    char* ws_base = nullptr;
    int64_t ws_bytes = 0;
    int *keys[2] = {nullptr, nullptr}, *vals[2] = {nullptr, nullptr};  // radix ping-pong, [max(M_max, cap_total)]
    int* table = nullptr;       // [bins * nw] per-wave digit counts / prefixes
    int* gtot = nullptr;        // [1024] per-digit totals
    int* tile_sums = nullptr;   // [tiles] flag counts per scan tile
    int* offsets = nullptr;     // [cap_u + 1] start row of each segment in sorted order
    int* seg_of_row = nullptr;  // [M_max] segment index of each sorted row
    int* uniq_ws = nullptr;     // [cap_u] copy of uniq of the current batch
    int* seg_slot = nullptr;    // [cap_u] buffer row of each segment; kSlotNew set = row is new, -1 = dropped
    int* scal = nullptr;        // [kSCount] device scalars, see enum Scalar
    int* long_list = nullptr;   // [tiles_seg] head tiles of the long segments of the current batch
    int* slot_of = nullptr;     // [N] buffer row of an ID, -1 = absent
    int* id_of_slot = nullptr;  // [cap_total]
    long long* cnt_of_slot = nullptr; // [cap_total] occurrences of the item of each row in the window
    float* G = nullptr;         // [cap_total, d] persistent per-item gradient
    float* E_ws = nullptr;      // [cap_u, d] representations when the caller passes E = NULL
    double* loss_part = nullptr; // [cap_chunk / kPseudoRows + 1] per-block sums of the pseudo-loss
    long long* cnt64 = nullptr; // [N] occurrences of each ID in the window (dense layout only)
    int* dense_sums = nullptr;  // [N / kScanTile + 1] items per tile of IDs (dense layout only)
    int* chunk_ids = nullptr;   // [cap_chunk] checked copy of a content-encoder batch's item IDs
    float* seg_first = nullptr; // [tiles_seg, d] partial sums of segments entering a tile
    float* seg_last = nullptr;  // [tiles_seg, d] partial sums of segments leaving a tile
    void* Wt = nullptr;         // [d, d_in] transposed weight (bf16 path)
    // two-layer encoder (cfg.d_hidden > 0) only:
    void* W1t = nullptr;        // [d_hidden, d_in] bf16
    void* W2t = nullptr;        // [d, d_hidden] bf16
    void* A1_ws = nullptr;      // [cap_u, d_hidden] bf16 activations when the caller keeps none
    int* iota = nullptr;        // [cap_chunk] 0, 1, 2, ...: row list of a matrix that needs no gather
    float* wg_partial = nullptr;// [splits, d_in, d] split-K partials of the weight gradient
    int wg_splits = 1;
    int num_cus = 256;          // compute units of the device (one contraction block each)

    // sorted order of the current batch (point into keys[]/vals[])
    int* sorted_keys = nullptr;
    int* perm = nullptr;

    // --- optional per-kernel event timing ---
    uint64_t prof_mask = 0;            // bit k set: time launches of kernel k
    std::vector<ProfSlot> prof_pool;   // events created once by gram_profile_enable
    size_t prof_used = 0;

    // --- host state ---
    bool have_unique = false;
    const int* last_uniq = nullptr;      // outputs of the most recent gram_unique (identity only)
    const int* last_inverse = nullptr;
    bool unique_consumed = false;  // the current batch was already accumulated
    bool window_imported = false;  // a saved state was merged into this window
    // The dedup of a batch also works out which buffer rows its items will get (seg_slot), from
    // the slot table as it is at that moment; gram_grad_accumulate commits them if the table has
    // not changed since (every change of it advances slot_epoch), else assigns rows afresh.
    uint64_t slot_epoch = 1;
    uint64_t prospect_epoch = 0;   // slot_epoch at which seg_slot was worked out; 0 = not at all
    int64_t cur_m = 0;
    int32_t steps_done = 0;
    int64_t window_positions = 0;  // positions accumulated in this window: bounds the buffer rows
    int* h_pinned = nullptr;    // [4] pinned host scratch for small read-backs
    std::string last_error;
};

// A kernel that uses more than 64 KiB of dynamic LDS needs its limit raised before its first
// launch on a device.  Raising it twice is harmless, so threads that race here only repeat the
// call; the flag is per kernel (template argument) and per device (bit).
template <auto Kernel>
inline void ensure_dynamic_lds(int bytes)
{
    static std::atomic<uint64_t> done{0};
    int dev = 0;
    (void)hipGetDevice(&dev);
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return;
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    done.fetch_or(bit, std::memory_order_release);
}

// Launch a kernel; with profiling enabled for `kid`, bracket it with two events
// on the same stream.
template <typename... KArgs, typename... Args>
inline void launch_smem(Ctx* c, int kid, void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t smem,
                        hipStream_t s, Args&&... args)
{
    ProfSlot* p = nullptr;
    if ((c->prof_mask >> kid) & 1u) {
        if (c->prof_used < c->prof_pool.size()) {
            p = &c->prof_pool[c->prof_used++];
            p->kid = kid;
            (void)hipEventRecord(p->start, s);
        }
    }
    hipLaunchKernelGGL(kernel, grid, block, smem, s, std::forward<Args>(args)...);
    if (p) (void)hipEventRecord(p->stop, s);
}

template <typename... KArgs, typename... Args>
inline void launch(Ctx* c, int kid, void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t s,
                   Args&&... args)
{
    launch_smem(c, kid, kernel, grid, block, 0, s, std::forward<Args>(args)...);
}

// ---- gram_sort.hip -------------------------------------------------------
SortPlan make_sort_plan(int key_bits, int64_t n_max);
// Stable LSD radix sort of (key, value) pairs on the low `key_bits` bits.
// keys_in: n keys (n = *n_dev if n_dev else n_host; n <= n_max).  vals_in may
// be NULL (value = index).  With check_range, keys outside [0, vocab_n) are
// replaced by `fix_key` and kErrBitRange is latched.  Results land in
// ctx->keys[r] / ctx->vals[r]; r is returned.
int radix_sort_pairs(Ctx* c, const int* keys_in, const int* vals_in, int n_host, const int* n_dev,
                     int64_t n_max, bool check_range, int fix_key, hipStream_t s);
void unique_from_sorted(Ctx* c, int n, int* uniq, int* inverse, int* counts, int* u_out, hipStream_t s,
                        bool prospect = false, int first_step = 0);
// One-launch dedup for small batches; returns false if n is too large for it.
bool unique_small(Ctx* c, const int* ids, int n, int fix_key, int* uniq, int* inverse, int* counts,
                  int* u_out, hipStream_t s, bool prospect = false, int first_step = 0);

// ---- gram_stream.hip -----------------------------------------------------
// H has the context's h_dtype (float32, or bf16 rounded to nearest even).
void gather_rows(Ctx* c, const float* E, const int* inverse, int64_t m, void* H, hipStream_t s);
void gather_heavy(Ctx* c, const float* E, int64_t m, void* H, hipStream_t s);
void pseudo_target(Ctx* c, const float* E, float* Ht, double* loss_dev, hipStream_t s);
// Checked copy of a content-encoder batch's IDs into c->chunk_ids and its size into scal[kSChunkN].
void chunk_ids_prepare(Ctx* c, const int* ids, int64_t n, hipStream_t s);
// With Ht: R[j,:] -= Ht[j,:] for the n rows of the batch in c->chunk_ids (zero for the padding
// item); without: R is taken as it is.  With loss_dev, 1/2 of the sum of the squares of R.
// R_bf16 (nullable, [n, d] bf16): also receives the miss rounded to bf16.
void pseudo_miss(Ctx* c, float* R, const float* Ht, int64_t n, double* loss_dev, hipStream_t s,
                 void* R_bf16 = nullptr);
void assign_slots(Ctx* c, hipStream_t s);
void segment_reduce(Ctx* c, const float* dH, int64_t m, hipStream_t s, bool commit = false);
void flush_export(Ctx* c, int* uniq_total, int* counts_total, long long* counts64_total, float* G_total,
                  int* u_total_dev, hipStream_t s);
const int* flush_meta_and_ranks(Ctx* c, int* uniq_total, int* counts_total, int* u_total_dev, hipStream_t s,
                                bool* left_to_caller);
void import_slots(Ctx* c, const int* ids, const long long* counts, const float* rows, int64_t n,
                  hipStream_t s);
void flush_dense(Ctx* c, int* uniq_total, int* counts_total, long long* counts64_total, float* G_total,
                 int* u_total_dev, hipStream_t s);
void import_dense(Ctx* c, const int* ids, const long long* counts, const float* rows, int64_t n,
                  hipStream_t s);
void fill_i32(int* p, int64_t n, int v, hipStream_t s);
void iota_i32(int* p, int64_t n, hipStream_t s);

// ---- gram_gemm.hip -------------------------------------------------------
// Returns true when H_scatter was given and the contraction's epilogue has already written H
// for every item with at most kLightMax positions (gather_heavy must follow); false when only E
// was written (gather_rows must follow).
// epi (bf16 contexts only; see the enum): what the contraction does with an output element
// before storing it; a mode other than kEpiPlain excludes the fused gather.
enum { kEpiPlain = 0, kEpiReluBf16 = 1, kEpiMinus = 2, kEpiGate = 3 };
bool encode_forward(Ctx* c, const void* X, const void* W, const int* uniq, const int* u_dev,
                    int64_t rows_max, float* E, hipStream_t s, void* H_scatter, bool caller_wants_E,
                    int epi = kEpiPlain, const void* aux = nullptr);
// Rows the weight gradient contracts over when they are not the persistent buffer's: row j pairs
// item ids[j] with rows[j,:] (float32, d columns); *n_dev rows are held, at most n_max.
// With d_in != 0 the contraction also takes its shape from here instead of the context: the
// matrix passed as X is [x_rows, d_in] (bf16), rows[] has d columns, dW is [d_in, d]; ids == NULL
// pairs rows[j] with row j of X; pad_id < 0: no row is skipped.
struct WgradRows {
    const int* ids;
    const float* rows;
    const int* n_dev;
    int64_t n_max;
    int64_t x_rows = 0;
    int d_in = 0, d = 0, pad_id = -1;
};
// Weight gradient over the buffer rows [first_row, first_row + n_rows) (clipped to the rows held),
// or over the rows of `other`, written to dW or added to it.
// export_G (buffer rows, bf16, whole window only): the kernel also writes buffer row s to
// export_G[rank_of_slot[s], :] (rank_of_slot NULL: to row s).  Returns false, and does not export,
// when that variant does not apply (float32 features, an operand beyond 4 GiB).
// meta (with export_G, one-step windows): the launch also exports IDs and counts and clears the slot map
struct WindowMeta {
    int* uniq_total;
    int* counts_total;
    int* u_total_dev;
};
bool encoder_wgrad(Ctx* c, const void* X, float* dW, hipStream_t s, int64_t first_row, int64_t n_rows,
                   bool accumulate, const WgradRows* other = nullptr, float* export_G = nullptr,
                   const int* rank_of_slot = nullptr, const WindowMeta* meta = nullptr);
// ---- gram_mlp.hip --------------------------------------------------------
// Forward of the two-layer encoder for the unique items of the batch; A1 (nullable) receives the
// bf16 hidden activations.  Return value as encode_forward.
bool mlp_forward(Ctx* c, const void* X, const void* W1, const void* W2, const int* uniq, const int* u_dev,
                 int64_t rows_max, void* A1, float* E, hipStream_t s, void* H_scatter, bool caller_wants_E);
int64_t mlp_batch_bytes(const Ctx* c, int64_t n);
// Backward of the two-layer encoder over the listed items from output-gradient rows (`rows`) or,
// with Ht, from the regression miss against stored targets (then loss_dev may receive Eq. 7).
void mlp_backward(Ctx* c, const void* X, const void* W1, const void* W2, const int* ids, const float* rows,
                  const float* Ht, int64_t n, void* work, float* dW1, float* dW2, bool accumulate,
                  double* loss_dev, hipStream_t s);

int wgrad_splits_for(const gram_config& cfg);
int wgrad_splits_dims(int d_in, int d, bool bf16);
// bf16 helpers the two-layer encoder shares with the linear one.
void transpose_weight(Ctx* c, const void* W, int rows, int cols, void* Wt, hipStream_t s);
// C[j,:] = epi(A[row_ids[j],:k] . Bt^T) for j < *n_dev (A bf16 [a_rows, k], Bt bf16 [n_out, k], C
// float32 [., n_out], or bf16 for kEpiReluBf16); a row whose ID equals pad_id is zero.  kEpiMinus
// subtracts the float32 matrix aux, kEpiGate keeps the value where the bf16 matrix aux is positive
// (both [., n_out]).  B_plain, if given, is the untransposed second operand [k, n_out]: where
// gemm_reads_plain_b says so, the kernels read it directly and Bt is not touched (the caller need
// not have filled it).
// Same return value and fused-gather rule as encode_forward.
bool gemm_reads_plain_b(const Ctx* c, int64_t rows_max, int64_t a_rows, int k, int n_out, int epi);
bool gemm_rows_bf16(Ctx* c, const void* A, int64_t a_rows, int k, const int* row_ids, int pad_id,
                    const int* n_dev, int64_t rows_max, const void* Bt, int n_out, float* C, hipStream_t s,
                    void* H_scatter, bool caller_wants_C, int epi = kEpiPlain, const void* aux = nullptr,
                    const void* B_plain = nullptr);

}  // namespace gram
