// Dedup of a batch of item IDs: the set B_I of unique items (Table 1 of the
// paper; Algorithm 1 ranges over it), its inverse index and multiplicities.
//
// Method: stable LSD radix sort of (id, position) pairs over only the
// ceil(log2 N) significant key bits, in digits of up to 10 bits (at most two
// passes for a vocabulary of a million items), followed by head-flag scan and
// compaction.  Each 64-lane wave owns a contiguous chunk of keys; ranks inside
// a wave come from ballot-based digit matching, ranks across blocks from a
// per-block digit table that one wave per digit prefix-sums.  Small batches
// take a one-launch variant that keeps everything in LDS (k_unique_small).
// All counters are integer (LDS atomics are order independent), so the result
// is exact.
#include "gram_internal.h"

namespace gram {

// Counters that a wave re-reads from LDS after its own lanes have written them are accessed
// through volatile pointers IN THE LDS ADDRESS SPACE: a volatile pointer without an address
// space is compiled to flat, system-coherent accesses, each followed by a wait for every
// outstanding memory operation of the wave (its scattered global stores included).
typedef __attribute__((address_space(3))) int lds_i32;
typedef __attribute__((address_space(3))) unsigned long long lds_u64;

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

// Exclusive scan of one value per thread over a 256-thread block; *total gets the block sum.
__device__ __forceinline__ int block_excl_scan(int v, int* total, int* sm /*[kWavesPerBlock]*/)
{
    const int incl = wave_incl_scan(v);
    if (lane_id() == kWave - 1) sm[wave_id()] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
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

constexpr int kSortBatch = 16;   // rounds whose keys are loaded ahead

// A block of 4 waves owns items * 256 consecutive keys; wave w of the block owns
// the w-th quarter of them.
SortPlan make_sort_plan(int key_bits, int64_t n_max)
{
    SortPlan p{};
    if (key_bits < 1) key_bits = 1;
    p.passes = (key_bits + kMaxDigitBits - 1) / kMaxDigitBits;
    int left = key_bits;
    for (int i = 0; i < p.passes; ++i) {
        int b = (left + (p.passes - i) - 1) / (p.passes - i);
        p.digit_bits[i] = b;
        left -= b;
    }
    // about 256 blocks (one per CU): the scatter pass issues two 4-byte stores per key to
    // unrelated addresses, and the rate of such stores per CU is what bounds it
    int64_t items = (n_max + (int64_t)kBlock * 256 - 1) / ((int64_t)kBlock * 256);
    if (items < 4) items = 4;
    if (items > 64) items = 64;
    p.items = (int)items;
    const int64_t kpb = (int64_t)kBlock * p.items;
    int64_t nb = (n_max + kpb - 1) / kpb;
    if (nb < 1) nb = 1;
    p.blocks = (int)nb;
    p.nw = p.blocks * kWavesPerBlock;
    return p;
}

// The keys of one wave's chunk are walked kSortBatch rounds of 64 keys at a time; the keys of a
// batch (and the values that travel with them: the expression VLOAD of the index idx_) are
// fetched together, because the rounds are short and otherwise each would wait for its own
// global load.  BODY sees the key k, its index idx, `valid` and the value vv.
#define GRAM_LOAD_BATCH(IT0, KB, VB, VLOAD)                                                         \
    _Pragma("unroll") for (int u = 0; u < kSortBatch; ++u) {                                        \
        const int64_t idx_ = base + (int64_t)((IT0) + u) * kWave + lane;                            \
        const bool in_ = (IT0) + u < items && idx_ < n;                                             \
        KB[u] = in_ ? keys_in[idx_] : 0;                                                            \
        VB[u] = in_ ? (VLOAD) : 0;                                                                  \
    }
#define GRAM_RUN_BATCH(IT0, KB, VB, BODY)                                                           \
    _Pragma("unroll") for (int u = 0; u < kSortBatch; ++u) {                                        \
        if ((IT0) + u >= items) break; /* wave-uniform */                                           \
        const int64_t idx = base + (int64_t)((IT0) + u) * kWave + lane;                             \
        const bool valid = idx < n;                                                                 \
        int k = KB[u];                                                                              \
        const int vv = VB[u];                                                                       \
        (void)vv;                                                                                   \
        BODY                                                                                        \
    }
#define GRAM_FOR_WAVE_KEYS(BODY)                                                                    \
    for (int it0 = 0; it0 < items; it0 += kSortBatch) {                                             \
        int kb_[kSortBatch], vb_[kSortBatch];                                                       \
        GRAM_LOAD_BATCH(it0, kb_, vb_, 0)                                                           \
        GRAM_RUN_BATCH(it0, kb_, vb_, BODY)                                                         \
    }
// The same walk with the first batch already in registers (KB0, VB0).
#define GRAM_FOR_WAVE_KEYS_FROM(KB0, VB0, VLOAD, BODY)                                              \
    for (int it0 = 0; it0 < items; it0 += kSortBatch) {                                             \
        int kb_[kSortBatch], vb_[kSortBatch];                                                       \
        if (it0 == 0) {                                                                             \
            _Pragma("unroll") for (int u = 0; u < kSortBatch; ++u) {                                \
                kb_[u] = KB0[u];                                                                    \
                vb_[u] = VB0[u];                                                                    \
            }                                                                                       \
        } else {                                                                                    \
            GRAM_LOAD_BATCH(it0, kb_, vb_, VLOAD)                                                   \
        }                                                                                           \
        GRAM_RUN_BATCH(it0, kb_, vb_, BODY)                                                         \
    }

// Digit histogram of one pass per block.  table[digit * nb + block] = count.
template <bool CHECK>
__global__ __launch_bounds__(kBlock) void k_radix_hist(const int* __restrict__ keys_in, int n_host,
                                                       const int* __restrict__ n_dev, int shift,
                                                       int dbits, int items,
                                                       int* __restrict__ table, int vocab_n,
                                                       int fix_key, int* __restrict__ err)
{
    __shared__ int cnt[1 << kMaxDigitBits];
    const int n = n_dev ? *n_dev : n_host;
    const int wave = wave_id(), lane = lane_id();
    const int bins = 1 << dbits;
    for (int b = threadIdx.x; b < bins; b += kBlock) cnt[b] = 0;
    __syncthreads();
    const int64_t base = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * items * kWave;
    bool bad = false;
    GRAM_FOR_WAVE_KEYS(
        if (valid) {
            if (CHECK && (k < 0 || k >= vocab_n)) { bad = true; k = fix_key; }
            atomicAdd(&cnt[(k >> shift) & (bins - 1)], 1);
        })
    if (CHECK && bad) atomicOr(err, kErrBitRange);
    __syncthreads();
    for (int b = threadIdx.x; b < bins; b += kBlock) table[(int64_t)b * gridDim.x + blockIdx.x] = cnt[b];
}

// One wave per digit: exclusive prefix over the blocks' counts (in place), digit total to gtot.
__global__ __launch_bounds__(kBlock) void k_radix_scan(int* __restrict__ table, int nb, int bins,
                                                       int* __restrict__ gtot)
{
    const int b = blockIdx.x * kWavesPerBlock + wave_id();
    if (b >= bins) return;
    const int lane = lane_id();
    int* row = table + (int64_t)b * nb;
    int carry = 0;
    // four chunks of 64 counts are fetched together: the scan of a chunk is short, and one chunk
    // per round trip would make the launch as long as its number of chunks
    for (int base = 0; base < nb; base += 4 * kWave) {
        int v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = base + u * kWave + lane;
            v[u] = i < nb ? row[i] : 0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = base + u * kWave + lane;
            const int incl = wave_incl_scan(v[u]);
            if (i < nb) row[i] = carry + incl - v[u];
            carry += __shfl(incl, kWave - 1);
        }
    }
    if (lane == 0) gtot[b] = carry;
}

// Stable scatter of one pass.  The block recounts its keys per wave, turns the counts into the
// first output slot of every (wave, digit), then each wave walks its chunk in rounds of 64 keys:
// lanes holding the same digit find each other with one ballot per digit bit and take consecutive
// slots in lane order.
template <bool CHECK>
__global__ __launch_bounds__(kBlock) void k_radix_scatter(
    const int* __restrict__ keys_in, const int* __restrict__ vals_in, int n_host,
    const int* __restrict__ n_dev, int shift, int dbits, int items,
    const int* __restrict__ table, const int* __restrict__ gtot, int* __restrict__ keys_out,
    int* __restrict__ vals_out, int vocab_n, int fix_key)
{
    __shared__ int digit_base[1 << kMaxDigitBits];
    __shared__ int cnt_s[kWavesPerBlock][1 << kMaxDigitBits];
    __shared__ int sm[kWavesPerBlock];
    const int n = n_dev ? *n_dev : n_host;
    const int wave = wave_id(), lane = lane_id();
    const int bins = 1 << dbits;
    const int64_t base = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * items * kWave;

    // Everything this block reads that does not depend on its own work is fetched first, in one
    // round trip: the first batch of its keys and values (kept for both walks below), its column
    // of the block table and the digit totals.
    int kb0[kSortBatch], vb0[kSortBatch];
    GRAM_LOAD_BATCH(0, kb0, vb0, (vals_in ? vals_in[idx_] : (int)idx_))
    static_assert((1 << kMaxDigitBits) <= 4 * kBlock, "a thread holds at most 4 digits of the block table");
    int tb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int b = threadIdx.x + i * kBlock;
        tb[i] = b < bins ? table[(int64_t)b * gridDim.x + blockIdx.x] : 0;
    }

    for (int b = threadIdx.x; b < bins; b += kBlock)
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) cnt_s[w][b] = 0;
    {   // exclusive scan of the digit totals, 4 digits per thread
        int v[4], s = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int b = threadIdx.x * 4 + i;
            v[i] = b < bins ? gtot[b] : 0;
            s += v[i];
        }
        int total;
        int run = block_excl_scan(s, &total, sm);      // contains barriers: cnt_s is zero after it
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int b = threadIdx.x * 4 + i;
            if (b < bins) digit_base[b] = run;
            run += v[i];
        }
    }
    GRAM_FOR_WAVE_KEYS_FROM(kb0, vb0, 0,
        if (valid) {
            if (CHECK && (k < 0 || k >= vocab_n)) k = fix_key;
            atomicAdd(&cnt_s[wave][(k >> shift) & (bins - 1)], 1);
        })
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int b = threadIdx.x + i * kBlock;
        if (b < bins) {
            int o = digit_base[b] + tb[i];
#pragma unroll
            for (int w = 0; w < kWavesPerBlock; ++w) {
                const int cw = cnt_s[w][b];
                cnt_s[w][b] = o;
                o += cw;
            }
        }
    }
    __syncthreads();

    volatile lds_i32* cnt = (volatile lds_i32*)cnt_s[wave];
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    GRAM_FOR_WAVE_KEYS_FROM(kb0, vb0, (vals_in ? vals_in[idx_] : (int)idx_),
        if (CHECK && valid && (k < 0 || k >= vocab_n)) k = fix_key;
        const int v = vv;
        const int dg = (k >> shift) & (bins - 1);
        unsigned long long peers = __ballot(valid);
        for (int bit = 0; bit < dbits; ++bit) {
            const bool one = (dg >> bit) & 1;
            const unsigned long long mm = __ballot(one);
            peers &= one ? mm : ~mm;
        }
        const int below = __popcll(peers & lt_mask);
        int pos = 0;
        if (valid) pos = cnt[dg] + below;
        __builtin_amdgcn_wave_barrier();
        if (valid && below == 0) cnt[dg] = pos + __popcll(peers);
        __builtin_amdgcn_wave_barrier();
        if (valid && (unsigned)pos < (unsigned)n) {     // pos < n always holds; the test keeps a
            keys_out[pos] = k;                           // logic error from becoming a stray store
            vals_out[pos] = v;
        })
}
#undef GRAM_FOR_WAVE_KEYS
#undef GRAM_FOR_WAVE_KEYS_FROM
#undef GRAM_LOAD_BATCH
#undef GRAM_RUN_BATCH

int radix_sort_pairs(Ctx* c, const int* keys_in, const int* vals_in, int n_host, const int* n_dev,
                     int64_t n_max, bool check_range, int fix_key, hipStream_t s)
{
    const SortPlan p = make_sort_plan(c->key_bits, n_max);
    const int* kin = keys_in;
    const int* vin = vals_in;
    int shift = 0, dst = 0;
    for (int pass = 0; pass < p.passes; ++pass) {
        const int db = p.digit_bits[pass];
        const int bins = 1 << db;
        const bool chk = check_range && pass == 0;
        if (chk)
            launch(c, KID_RADIX_HIST, k_radix_hist<true>, dim3(p.blocks), dim3(kBlock), s, kin, n_host,
                               n_dev, shift, db, p.items, c->table, c->cfg.vocab_n, fix_key,
                               c->scal + kSErr);
        else
            launch(c, KID_RADIX_HIST, k_radix_hist<false>, dim3(p.blocks), dim3(kBlock), s, kin, n_host,
                               n_dev, shift, db, p.items, c->table, 0, 0, c->scal + kSErr);
        launch(c, KID_RADIX_SCAN, k_radix_scan, dim3((bins + kWavesPerBlock - 1) / kWavesPerBlock),
               dim3(kBlock), s, c->table, p.blocks, bins, c->gtot);
        if (chk)
            launch(c, KID_RADIX_SCATTER, k_radix_scatter<true>, dim3(p.blocks), dim3(kBlock), s, kin, vin,
                               n_host, n_dev, shift, db, p.items, c->table, c->gtot,
                               c->keys[dst], c->vals[dst], c->cfg.vocab_n, fix_key);
        else
            launch(c, KID_RADIX_SCATTER, k_radix_scatter<false>, dim3(p.blocks), dim3(kBlock), s, kin, vin,
                               n_host, n_dev, shift, db, p.items, c->table, c->gtot,
                               c->keys[dst], c->vals[dst], 0, 0);
        kin = c->keys[dst];
        vin = c->vals[dst];
        shift += db;
        dst ^= 1;
    }
    return dst ^ 1;
}

// ---- head flags -> uniq / inverse / offsets / counts / prospective buffer rows ----

__device__ __forceinline__ bool is_head(const int* __restrict__ sk, int r)
{
    return r == 0 || sk[r] != sk[r - 1];
}

// Two launches over tiles of kScanTile sorted rows.  The first leaves three figures per tile
// (tile_info[t], [T + t], [2 T + t] with T tiles): the number of segment heads in the tile, how
// many of those items have no row in the window's buffer yet, and the row of the tile's first
// head (-1: none).  The second turns them into everything that is known per unique item:
// uniq, offsets, counts (a head's segment ends at the next head, which may lie tiles ahead: the
// third figure finds it), the inverse index, and - when the context keeps a slot table - the
// buffer row each item WOULD get from the next gram_grad_accumulate (seg_slot: its row, or for
// an item new to the window the next free row with kSlotNew set, in ascending-ID order, or -1
// when the buffer is full).  Nothing of the slot table is written here: the accumulate step
// commits those rows, provided the table has not changed in between.
__device__ __forceinline__ int block_min(int v, int* sm)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        const int t = __shfl_down(v, o);
        v = t < v ? t : v;
    }
    if (lane_id() == 0) sm[wave_id()] = v;
    __syncthreads();
    int m = sm[0];
#pragma unroll
    for (int w = 1; w < kWavesPerBlock; ++w) m = sm[w] < m ? sm[w] : m;
    __syncthreads();
    return m;
}

constexpr int kNoRow = 0x7fffffff;

__global__ __launch_bounds__(kBlock) void k_heads_count(const int* __restrict__ sk, int n,
                                                        const int* __restrict__ slot_of,
                                                        int* __restrict__ tile_info, int first_step)
{
    __shared__ int sm[kWavesPerBlock];
    const int r0 = blockIdx.x * kScanTile + threadIdx.x * 4;
    int s = 0, fresh = 0, first = kNoRow;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (r0 + i < n && is_head(sk, r0 + i)) {
            ++s;
            if (first == kNoRow) first = r0 + i;
            // (in the first step of a window the buffer holds nothing: every item is new)
            if (slot_of && (first_step || slot_of[sk[r0 + i]] < 0)) ++fresh;
        }
    const int tot = block_sum(s, sm);
    const int tot_fresh = block_sum(fresh, sm);
    const int row = block_min(first, sm);
    if (threadIdx.x == 0) {
        tile_info[blockIdx.x] = tot;
        tile_info[gridDim.x + blockIdx.x] = tot_fresh;
        tile_info[2 * gridDim.x + blockIdx.x] = row == kNoRow ? -1 : row;
    }
}

__global__ __launch_bounds__(kBlock) void k_heads_emit(
    const int* __restrict__ sk, const int* __restrict__ sv, int n, const int* __restrict__ tile_info,
    int* __restrict__ uniq, int* __restrict__ inverse, int* __restrict__ counts,
    int* __restrict__ offsets, int* __restrict__ seg_of_row, int* __restrict__ uniq_ws,
    int* __restrict__ u_out, const int* __restrict__ slot_of, int* __restrict__ seg_slot,
    int* __restrict__ scal, int first_step, int cap_total)
{
    __shared__ int sm[kWavesPerBlock];
    __shared__ int s_rows[kScanTile + 1];     // rows of the tile's heads, then the next head's row
    __shared__ int s_next;
    const int T = gridDim.x;
    // Everything that does not depend on this block's own work is fetched before the first
    // barrier, in one round trip: the thread's 4 sorted keys and positions, the key before them,
    // the figures of the tiles before and (a first look) after this one, the buffer's row count.
    const int r0 = blockIdx.x * kScanTile + threadIdx.x * 4;
    int key[4] = {0, 0, 0, 0}, posn[4] = {0, 0, 0, 0};
    if (r0 + 3 < n) {           // whole groups of 4: 16-byte loads (the arrays are 256-byte aligned)
        const int4 k4 = *reinterpret_cast<const int4*>(sk + r0);
        const int4 p4 = *reinterpret_cast<const int4*>(sv + r0);
        key[0] = k4.x; key[1] = k4.y; key[2] = k4.z; key[3] = k4.w;
        posn[0] = p4.x; posn[1] = p4.y; posn[2] = p4.z; posn[3] = p4.w;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (r0 + i < n) {
                key[i] = sk[r0 + i];
                posn[i] = sv[r0 + i];
            }
    }
    const int prev = (r0 > 0 && r0 < n) ? sk[r0 - 1] : -1;
    const int u_base = (slot_of && !first_step) ? scal[kSUTotal] : 0;   // a flush leaves the old count behind
    const int ahead0 = (int)blockIdx.x + 1 + (int)threadIdx.x < T ? tile_info[2 * T + blockIdx.x + 1 + threadIdx.x] : -1;
    int pre = 0, pre_fresh = 0;
    for (int t = threadIdx.x; t < (int)blockIdx.x; t += kBlock) {
        pre += tile_info[t];
        pre_fresh += tile_info[T + t];
    }
    bool f[4];
    int old[4];
    int s = 0, fresh = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[i] = (r0 + i < n) && (r0 + i == 0 || key[i] != (i ? key[i - 1] : prev));
        old[i] = 0;
        s += f[i] ? 1 : 0;
        if (f[i] && slot_of) {
            old[i] = first_step ? -1 : slot_of[key[i]];
            fresh += old[i] < 0 ? 1 : 0;
        }
    }
    pre = block_sum(pre, sm);
    pre_fresh = block_sum(pre_fresh, sm);
    if (threadIdx.x == 0) s_next = kNoRow;
    int total, total_fresh;
    const int local = block_excl_scan(s, &total, sm);
    const int local_fresh = block_excl_scan(fresh, &total_fresh, sm);
    {
        int li = local;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (f[i]) s_rows[li++] = r0 + i;
    }
    // the first head after this tile: the tiles ahead are looked at kBlock at a time (their first
    // heads ascend with the tile index, so the minimum is the nearest)
    for (int base = blockIdx.x + 1; base < T; base += kBlock) {
        const int t = base + threadIdx.x;
        const int row = base == (int)blockIdx.x + 1 ? ahead0 : (t < T ? tile_info[2 * T + t] : -1);
        if (row >= 0) atomicMin(&s_next, row);
        __syncthreads();
        if (s_next != kNoRow) break;           // the same value for every thread
        __syncthreads();
    }
    __syncthreads();
    if (threadIdx.x == 0) s_rows[total] = s_next == kNoRow ? n : s_next;
    __syncthreads();

    int run = pre + local, li = local, next_slot = u_base + pre_fresh + local_fresh;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = r0 + i;
        if (r < n) {
            run += f[i] ? 1 : 0;
            const int seg = run - 1;
            seg_of_row[r] = seg;
            inverse[posn[i]] = seg;
            if (f[i]) {
                uniq[seg] = key[i];
                uniq_ws[seg] = key[i];
                offsets[seg] = r;
                counts[seg] = s_rows[li + 1] - r;
                ++li;
                if (slot_of) {
                    int code = old[i];
                    if (code < 0) {
                        const int slot = next_slot++;
                        code = slot < cap_total ? (slot | kSlotNew) : -1;
                    }
                    seg_slot[seg] = code;
                }
            }
        }
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        const int u = pre + total;
        scal[kSU] = u;
        if (u_out) *u_out = u;
        offsets[u] = n;
        if (slot_of) {
            const int nt = u_base + pre_fresh + total_fresh;
            scal[kSUNext] = nt < cap_total ? nt : cap_total;
            scal[kSLongCount] = 0;
        }
    }
}

__global__ void k_unique_empty(int* u_ws, int* u_out, int* offsets)
{
    if (threadIdx.x == 0) {
        *u_ws = 0;
        if (u_out) *u_out = 0;
        offsets[0] = 0;
    }
}

// ---- small batches: the whole dedup in one block ------------------------------------
//
// Up to kSmallMaxN positions: keys and positions live in LDS, the radix passes
// (8-bit digits, 16 waves), the head-flag scan and the compaction all run in one launch
// of 1024 threads.  A step of the paper-shaped KT and news batches moves a few
// microseconds of HBM traffic, so its cost is the number of launches - and, inside this
// one block, the number of instructions its 16 waves issue on one CU:
//  * the lanes of a wave that hold the same digit find each other through a per-wave table
//    of 64-bit lane masks in LDS (one atomic OR and one read per round; the first lane of a
//    group clears the entry again) instead of one ballot per digit bit;
//  * positions are 16-bit, which makes room for that table;
//  * `inverse` is assembled in LDS and written in position order, because a CU retires
//    scattered 4-byte stores at about one lane per clock.
constexpr int kSmallThreads = 1024;
constexpr int kSmallWaves = kSmallThreads / kWave;
constexpr int kSmallMaxN = 8192;
constexpr int kSmallBits = 8;
constexpr int kSmallBins = 1 << kSmallBits;
constexpr int kSmallRounds = kSmallMaxN / kSmallWaves / kWave;   // rounds of 64 keys per wave, at most
// LDS, in ints: keys x2 | positions x2 (16-bit) | per-wave digit counts | per-wave peer masks (64-bit) | wave sums
constexpr int kSmallOffV = 2 * kSmallMaxN;
constexpr int kSmallOffCnt = kSmallOffV + kSmallMaxN;
constexpr int kSmallOffPeer = kSmallOffCnt + kSmallWaves * kSmallBins;
constexpr int kSmallOffSum = kSmallOffPeer + 2 * kSmallWaves * kSmallBins;
constexpr size_t kSmallLds = (size_t)(kSmallOffSum + 2 * kSmallWaves) * sizeof(int);
static_assert(2 * kSmallWaves * kSmallBins >= kSmallMaxN, "the peer table doubles as the segment-start list");

// Exclusive scan of one value per thread over the 1024-thread block.
__device__ __forceinline__ int block1024_excl_scan(int v, int* total, int* wsum /*[2*kSmallWaves]*/)
{
    const int incl = wave_incl_scan(v);
    if (lane_id() == kWave - 1) wsum[wave_id()] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kSmallWaves; ++w) {
        const int t = wsum[w];
        if (w < wave_id()) base += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return base + incl - v;
}

__global__ __launch_bounds__(kSmallThreads) void k_unique_small(
    const int* __restrict__ ids, int n, int key_bits, int vocab_n, int fix_key, int* __restrict__ err,
    int* __restrict__ sorted_keys, int* __restrict__ perm, int* __restrict__ uniq,
    int* __restrict__ inverse, int* __restrict__ counts, int* __restrict__ offsets,
    int* __restrict__ seg_of_row, int* __restrict__ uniq_ws, int* __restrict__ u_ws,
    int* __restrict__ u_out, const int* __restrict__ slot_of, int* __restrict__ seg_slot,
    int* __restrict__ scal, int first_step, int cap_total)
{
    extern __shared__ __attribute__((aligned(16))) int lds[];
    // keys of order `o` at KBUF(o), positions at VBUF(o)
#define KBUF(o) (lds + (o) * kSmallMaxN)
#define VBUF(o) (reinterpret_cast<uint16_t*>(lds + kSmallOffV) + (o) * kSmallMaxN)
    int* cnt_all = lds + kSmallOffCnt;                   // [kSmallWaves][kSmallBins]
    unsigned long long* peer_all = reinterpret_cast<unsigned long long*>(lds + kSmallOffPeer);
    int* wsum = lds + kSmallOffSum;
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();

    bool bad = false;
    for (int i = tid; i < n; i += kSmallThreads) {
        int k = ids[i];
        if (k < 0 || k >= vocab_n) { bad = true; k = fix_key; }
        KBUF(0)[i] = k;
        VBUF(0)[i] = (uint16_t)i;
    }
    if (bad) atomicOr(err, kErrBitRange);
    for (int b = tid; b < kSmallWaves * kSmallBins; b += kSmallThreads) peer_all[b] = 0ull;
    __syncthreads();

    // wave w owns the contiguous chunk [w * cw, (w + 1) * cw) of the current order
    const int cw = ((n + kSmallWaves - 1) / kSmallWaves + kWave - 1) / kWave * kWave;
    const int cbeg = wave * cw;
    const int cend = cbeg + cw < n ? cbeg + cw : n;
    volatile lds_i32* cnt = (volatile lds_i32*)(cnt_all + wave * kSmallBins);
    volatile lds_u64* peer = (volatile lds_u64*)(peer_all + wave * kSmallBins);
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    int cur = 0;
    for (int shift = 0; shift < key_bits; shift += kSmallBits) {
        for (int b = lane; b < kSmallBins; b += kWave) cnt[b] = 0;
        __syncthreads();
        // the keys (and, for the second walk, positions) of all of the wave's rounds are read from
        // LDS up front: a round is a chain of dependent LDS operations, and the reads of the next
        // round would otherwise wait behind it
        int kr[kSmallRounds];
#pragma unroll
        for (int r = 0; r < kSmallRounds; ++r) {
            const int i = cbeg + r * kWave + lane;
            kr[r] = i < cend ? KBUF(cur)[i] : 0;
        }
#pragma unroll
        for (int r = 0; r < kSmallRounds; ++r) {
            if (cbeg + r * kWave >= cend) break;             // wave-uniform
            const bool valid = cbeg + r * kWave + lane < cend;
            const int dg = valid ? (kr[r] >> shift) & (kSmallBins - 1) : -1;
            // the digit of the round's first key is counted once for all lanes that hold it:
            // padding and very popular items would otherwise pile up on one LDS counter
            const int d0 = __builtin_amdgcn_readfirstlane(dg);
            const unsigned long long m0 = __ballot(dg == d0);
            if (lane == 0) atomicAdd(&cnt_all[wave * kSmallBins + d0], (int)__popcll(m0));
            else if (valid && dg != d0) atomicAdd(&cnt_all[wave * kSmallBins + dg], 1);
        }
        __syncthreads();
        {   // exclusive scan in (digit, wave) order; thread t owns digit t / 4, waves 4 (t % 4) .. + 3
            const int dg = tid >> 2, w0 = (tid & 3) * 4;
            int v[4], sum = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = cnt_all[(w0 + i) * kSmallBins + dg];
                sum += v[i];
            }
            int total;
            int run = block1024_excl_scan(sum, &total, wsum);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                cnt_all[(w0 + i) * kSmallBins + dg] = run;
                run += v[i];
            }
        }
        __syncthreads();
        int vr[kSmallRounds];
#pragma unroll
        for (int r = 0; r < kSmallRounds; ++r) {
            const int i = cbeg + r * kWave + lane;
            vr[r] = i < cend ? VBUF(cur)[i] : 0;
        }
#pragma unroll
        for (int r = 0; r < kSmallRounds; ++r) {
            if (cbeg + r * kWave >= cend) break;             // wave-uniform
            const bool valid = cbeg + r * kWave + lane < cend;
            const int k = kr[r];
            const int v = vr[r];
            const int dg = (k >> shift) & (kSmallBins - 1);
            // Lanes holding the digit of the round's first key know their group from one ballot
            // (padding and very popular items fill most of a round); the others meet through the
            // mask table.  LDS operations of one wave execute in program order: every lane's OR
            // lands before the reads below, and every lane has read before a group's first lane
            // writes.
            const int d0 = __builtin_amdgcn_readfirstlane(dg);
            const unsigned long long m0 = __ballot(valid && dg == d0);
            const bool in0 = valid && dg == d0;
            if (valid && !in0) atomicOr(&peer_all[wave * kSmallBins + dg], 1ull << lane);
            __builtin_amdgcn_wave_barrier();
            unsigned long long peers = 0ull;
            int pos = 0;
            if (valid) {
                peers = in0 ? m0 : peer[dg];
                pos = cnt[dg];
            }
            const int below = __popcll(peers & lt_mask);
            pos += below;
            __builtin_amdgcn_wave_barrier();
            if (valid && below == 0) {
                cnt[dg] = pos + __popcll(peers);
                if (!in0) peer[dg] = 0ull;
            }
            __builtin_amdgcn_wave_barrier();
            if (valid && (unsigned)pos < (unsigned)n) {
                KBUF(cur ^ 1)[pos] = k;
                VBUF(cur ^ 1)[pos] = (uint16_t)v;
            }
        }
        __syncthreads();
        cur ^= 1;
    }

    // head flags and their scan: thread t owns the 8 sorted rows 8 t .. 8 t + 7 and leaves each
    // row's segment index in LDS; the outputs are then written with consecutive threads on
    // consecutive rows / positions, so that the stores of a wave coalesce
    const int* sk = KBUF(cur);
    const uint16_t* sv = VBUF(cur);
    int* lseg = KBUF(cur ^ 1);                               // free after the last pass: segment of every sorted row
    int* loff = reinterpret_cast<int*>(peer_all);            // first sorted row of every segment
    uint16_t* linv = VBUF(cur ^ 1);                          // segment of every position
    const int r0 = tid * 8;
    // the thread's 8 keys and positions as 16-byte LDS reads (rows 8 t .. 8 t + 7 one by one
    // would hit the same banks in every lane)
    int key[8];
    uint16_t posn[8];
    {
        const int4 k0 = *reinterpret_cast<const int4*>(sk + r0);
        const int4 k1 = *reinterpret_cast<const int4*>(sk + r0 + 4);
        key[0] = k0.x; key[1] = k0.y; key[2] = k0.z; key[3] = k0.w;
        key[4] = k1.x; key[5] = k1.y; key[6] = k1.z; key[7] = k1.w;
        const uint4 p4 = *reinterpret_cast<const uint4*>(sv + r0);
        posn[0] = (uint16_t)p4.x; posn[1] = (uint16_t)(p4.x >> 16); posn[2] = (uint16_t)p4.y; posn[3] = (uint16_t)(p4.y >> 16);
        posn[4] = (uint16_t)p4.z; posn[5] = (uint16_t)(p4.z >> 16); posn[6] = (uint16_t)p4.w; posn[7] = (uint16_t)(p4.w >> 16);
    }
    const int prev = r0 > 0 && r0 < n ? sk[r0 - 1] : -1;
    bool f[8];
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = r0 + i;
        f[i] = r < n && (r == 0 || key[i] != (i ? key[i - 1] : prev));
        sum += f[i] ? 1 : 0;
    }
    int total;
    int run = block1024_excl_scan(sum, &total, wsum);
    int seg8[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = r0 + i;
        run += f[i] ? 1 : 0;
        seg8[i] = run - 1;
        if (r < n) {
            linv[posn[i]] = (uint16_t)(run - 1);
            if (f[i]) loff[run - 1] = r;
        }
    }
    if (r0 < n) {       // rows past n inside the last thread's 8 are never read back
        *reinterpret_cast<int4*>(lseg + r0) = make_int4(seg8[0], seg8[1], seg8[2], seg8[3]);
        *reinterpret_cast<int4*>(lseg + r0 + 4) = make_int4(seg8[4], seg8[5], seg8[6], seg8[7]);
    }
    if (tid == 0) {
        *u_ws = total;
        if (u_out) *u_out = total;
        offsets[total] = n;
    }
    __syncthreads();
    for (int r = tid; r < n; r += kSmallThreads) {
        sorted_keys[r] = sk[r];
        perm[r] = sv[r];
        seg_of_row[r] = lseg[r];
        inverse[r] = linv[r];
    }
    for (int j = tid; j < total; j += kSmallThreads) {
        const int r = loff[j];
        const int key = sk[r];
        uniq[j] = key;
        uniq_ws[j] = key;
        offsets[j] = r;
        counts[j] = (j + 1 < total ? loff[j + 1] : n) - r;
    }
    // the buffer rows the items would get from the next gram_grad_accumulate (see k_heads_emit):
    // thread t looks up items 8 t .. 8 t + 7, one scan ranks the items new to the window
    if (slot_of) {
        const int j0 = tid * 8;
        int old[8], fresh = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            old[i] = 0;
            if (j0 + i < total) {
                // in the first step of a window the buffer holds nothing: every item is new
                old[i] = first_step ? -1 : slot_of[sk[loff[j0 + i]]];
                fresh += old[i] < 0 ? 1 : 0;
            }
        }
        int total_fresh;
        const int u_base = first_step ? 0 : scal[kSUTotal];    // a flush leaves the old count behind
        int next_slot = u_base + block1024_excl_scan(fresh, &total_fresh, wsum);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (j0 + i < total) {
                int code = old[i];
                if (code < 0) {
                    const int slot = next_slot++;
                    code = slot < cap_total ? (slot | kSlotNew) : -1;
                }
                seg_slot[j0 + i] = code;
            }
        if (tid == 0) {
            const int nt = u_base + total_fresh;
            scal[kSUNext] = nt < cap_total ? nt : cap_total;
            scal[kSLongCount] = 0;
        }
    }
#undef KBUF
#undef VBUF
}

// prospect: also work out the buffer rows the items would get (slot-table contexts only);
// first_step: the window's buffer holds nothing yet.
void unique_from_sorted(Ctx* c, int n, int* uniq, int* inverse, int* counts, int* u_out,
                        hipStream_t s, bool prospect, int first_step)
{
    if (n == 0) {
        launch(c, KID_UNIQUE_EMPTY, k_unique_empty, dim3(1), dim3(kWave), s, c->scal + kSU, u_out, c->offsets);
        return;
    }
    const int tiles = (n + kScanTile - 1) / kScanTile;
    const int* slot_of = prospect ? c->slot_of : nullptr;
    launch(c, KID_HEADS_COUNT, k_heads_count, dim3(tiles), dim3(kBlock), s, c->sorted_keys, n, slot_of,
           c->tile_sums, first_step);
    launch(c, KID_HEADS_EMIT, k_heads_emit, dim3(tiles), dim3(kBlock), s, c->sorted_keys, c->perm, n,
           c->tile_sums, uniq, inverse, counts, c->offsets, c->seg_of_row, c->uniq_ws, u_out, slot_of,
           c->seg_slot, c->scal, first_step, (int)c->cap_total);
}

bool unique_small(Ctx* c, const int* ids, int n, int fix_key, int* uniq, int* inverse, int* counts,
                  int* u_out, hipStream_t s, bool prospect, int first_step)
{
    if (n <= 0 || n > kSmallMaxN) return false;
    ensure_dynamic_lds<k_unique_small>((int)kSmallLds);
    c->sorted_keys = c->keys[0];
    c->perm = c->vals[0];
    launch_smem(c, KID_UNIQUE_SMALL, k_unique_small, dim3(1), dim3(kSmallThreads), kSmallLds, s, ids, n,
                c->key_bits, c->cfg.vocab_n, fix_key, c->scal + kSErr, c->sorted_keys, c->perm, uniq, inverse,
                counts, c->offsets, c->seg_of_row, c->uniq_ws, c->scal + kSU, u_out,
                prospect ? c->slot_of : nullptr, c->seg_slot, c->scal, first_step, (int)c->cap_total);
    return true;
}

}  // namespace gram
