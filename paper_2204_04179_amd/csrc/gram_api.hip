// C ABI of libgram (see include/gram.h): argument checks, call-order checks,
// workspace layout, kernel sequencing.  No arithmetic of the method lives here.
#include <stdarg.h>
#include <stdio.h>

#include <mutex>
#include <new>

#include "gram_internal.h"

using namespace gram;

namespace {

std::string g_create_error;

int fail(Ctx* c, int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->last_error = buf; else g_create_error = buf;
    return code;
}

int hip_fail(Ctx* c, hipError_t e, const char* what)
{
    return fail(c, GRAM_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

int bits_for(int32_t vocab_n)
{
    int b = 1;
    while (b < 31 && ((int64_t)1 << b) < (int64_t)vocab_n) ++b;
    return b;
}

int64_t table_elems_for(int64_t n_sort_max)
{
    // Upper bound, over every n <= n_sort_max, of the digit table make_sort_plan(n) needs: its blocks
    // hold at least 1024 and at most 256 * 64 keys each, and there are at most 256 of them until the
    // keys per block reach that maximum.
    int64_t nb = (n_sort_max + 1023) / 1024;
    if (nb > 256) {
        nb = (n_sort_max + 16383) / 16384;
        if (nb < 256) nb = 256;
    }
    return ((int64_t)1 << kMaxDigitBits) * (nb + 1);
}

struct Derived {
    int64_t cap_u, cap_total, cap_chunk, n_sort_max, tiles_scan, tiles_seg;
    int splits;
};

const char* validate(const gram_config* cfg, Derived* dv)
{
    if (!cfg) return "cfg is NULL";
    if (cfg->vocab_n < 1) return "vocab_n must be >= 1";
    if (cfg->xw_dtype != GRAM_F32 && cfg->xw_dtype != GRAM_BF16) return "xw_dtype must be GRAM_F32 or GRAM_BF16";
    if (cfg->d_in < 1 || (cfg->xw_dtype == GRAM_BF16 && cfg->d_in % 8 != 0))
        return "d_in must be positive (a multiple of 8 for bf16)";
    if (cfg->d < 4 || cfg->d % 4 != 0) return "d must be a positive multiple of 4";
    if (cfg->max_positions < 1 || cfg->max_positions > ((int64_t)1 << 30))
        return "max_positions must be in [1, 2^30]";
    if (cfg->k_steps < 1) return "k_steps must be >= 1";
    if (cfg->pad_id >= cfg->vocab_n) return "pad_id must be < vocab_n (negative = no padding)";
    if (cfg->u_total_cap < 0) return "u_total_cap must be >= 0";
    if (cfg->buffer_layout != GRAM_BUFFER_SLOTS && cfg->buffer_layout != GRAM_BUFFER_DENSE)
        return "buffer_layout must be GRAM_BUFFER_SLOTS or GRAM_BUFFER_DENSE";
    if (cfg->h_dtype != GRAM_F32 && cfg->h_dtype != GRAM_BF16) return "h_dtype must be GRAM_F32 or GRAM_BF16";
    if (cfg->d_hidden < 0) return "d_hidden must be >= 0 (0 = linear encoder)";
    if (cfg->d_hidden > 0 && (cfg->xw_dtype != GRAM_BF16 || cfg->d_hidden % 8 != 0 || cfg->d % 8 != 0))
        return "the two-layer encoder needs bf16 features and d_hidden, d multiples of 8";
    const bool dense = cfg->buffer_layout == GRAM_BUFFER_DENSE;
    if (dense && cfg->u_total_cap != 0 && cfg->u_total_cap != cfg->vocab_n)
        return "the dense buffer has one row per ID: u_total_cap must be 0 or vocab_n";
    dv->cap_u = cfg->max_positions < cfg->vocab_n ? cfg->max_positions : cfg->vocab_n;
    int64_t km = (int64_t)cfg->k_steps * cfg->max_positions;
    dv->cap_total = cfg->u_total_cap ? cfg->u_total_cap : (km < cfg->vocab_n ? km : cfg->vocab_n);
    if (dense) dv->cap_total = cfg->vocab_n;
    if (dv->cap_total >= ((int64_t)1 << 30)) return "persistent buffer rows must be < 2^30";
    dv->cap_chunk = dv->cap_u > dv->cap_total ? dv->cap_u : dv->cap_total;
    dv->n_sort_max = cfg->max_positions > dv->cap_total ? cfg->max_positions : dv->cap_total;
    dv->tiles_scan = (cfg->max_positions + kScanTile - 1) / kScanTile + 1;
    dv->tiles_seg = (cfg->max_positions + kSegRows - 1) / kSegRows;
    dv->splits = wgrad_splits_for(*cfg);
    return nullptr;
}

// Carves the single device allocation; with base == nullptr only measures.
int64_t layout(Ctx* c, const gram_config& cfg, const Derived& dv, char* base)
{
    int64_t off = 0;
    auto take = [&](int64_t bytes) -> char* {
        char* p = base ? base + off : nullptr;
        off += align_up(bytes > 0 ? bytes : 1, 256);
        return p;
    };
    const int64_t d = cfg.d, d_in = cfg.d_in;
    int* scal = (int*)take(64 * sizeof(int));
    int* keys0 = (int*)take(dv.n_sort_max * 4);
    int* keys1 = (int*)take(dv.n_sort_max * 4);
    int* vals0 = (int*)take(dv.n_sort_max * 4);
    int* vals1 = (int*)take(dv.n_sort_max * 4);
    int* table = (int*)take(table_elems_for(dv.n_sort_max) * 4);
    int* gtot = (int*)take((1 << kMaxDigitBits) * 4);
    int* tile_sums = (int*)take(dv.tiles_scan * 3 * 4);     // three figures per scan tile
    int* offsets = (int*)take((dv.cap_u + 2) * 4);
    int* seg_of_row = (int*)take(cfg.max_positions * 4);
    int* uniq_ws = (int*)take(dv.cap_u * 4);
    int* seg_slot = (int*)take(dv.cap_u * 4);
    int* long_list = (int*)take(dv.tiles_seg * 4);
    const bool dense = cfg.buffer_layout == GRAM_BUFFER_DENSE;
    int* slot_of = (int*)take(dense ? 1 : (int64_t)cfg.vocab_n * 4);
    int* id_of_slot = (int*)take(dense ? 1 : dv.cap_total * 4);
    long long* cnt_of_slot = (long long*)take(dense ? 1 : dv.cap_total * 8);
    long long* cnt64 = (long long*)take(dense ? (int64_t)cfg.vocab_n * 8 : 1);
    int* dense_sums = (int*)take(dense ? ((int64_t)cfg.vocab_n / kScanTile + 2) * 4 : 1);
    float* G = (float*)take(dv.cap_total * d * 4);
    float* E_ws = (float*)take(dv.cap_u * d * 4);
    double* loss_part = (double*)take((dv.cap_chunk / kPseudoRows + 1) * 8);
    int* chunk_ids = (int*)take(dv.cap_chunk * 4);
    float* seg_first = (float*)take(dv.tiles_seg * d * 4);
    float* seg_last = (float*)take(dv.tiles_seg * d * 4);
    void* Wt = take(cfg.xw_dtype == GRAM_BF16 ? d * d_in * 2 : 1);
    const int64_t dh = cfg.d_hidden;
    int64_t partial_elems = (int64_t)dv.splits * d_in * d;
    if (dh > 0) {
        const int64_t bottom = (int64_t)wgrad_splits_dims((int)d_in, (int)dh, true) * d_in * dh;
        const int64_t top = (int64_t)wgrad_splits_dims((int)dh, (int)d, true) * dh * d;
        if (bottom > partial_elems) partial_elems = bottom;
        if (top > partial_elems) partial_elems = top;
    }
    float* wg_partial = (float*)take(partial_elems * 4);
    void* W1t = take(dh > 0 ? dh * d_in * 2 : 1);
    void* W2t = take(dh > 0 ? d * dh * 2 : 1);
    void* A1_ws = take(dh > 0 ? dv.cap_u * dh * 2 : 1);
    int* iota = (int*)take(dh > 0 ? dv.cap_chunk * 4 : 1);
    if (c && base) {
        c->scal = scal; c->keys[0] = keys0; c->keys[1] = keys1; c->vals[0] = vals0; c->vals[1] = vals1;
        c->table = table; c->gtot = gtot; c->tile_sums = tile_sums; c->offsets = offsets;
        c->seg_of_row = seg_of_row; c->uniq_ws = uniq_ws; c->seg_slot = seg_slot;
        c->long_list = long_list; c->slot_of = slot_of; c->id_of_slot = dense ? nullptr : id_of_slot;
        c->cnt_of_slot = cnt_of_slot; c->cnt64 = cnt64; c->dense_sums = dense_sums; c->G = G; c->E_ws = E_ws; c->loss_part = loss_part; c->chunk_ids = chunk_ids; c->seg_first = seg_first;
        c->seg_last = seg_last; c->Wt = Wt; c->wg_partial = wg_partial;
        c->W1t = W1t; c->W2t = W2t; c->A1_ws = A1_ws; c->iota = iota;
    }
    return off;
}

int launch_status(Ctx* c, const char* what)
{
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? GRAM_OK : hip_fail(c, e, what);
}

// Copy the device scalars to the host, wait, and turn latched error bits into a status.
int sync_scalars(Ctx* c, hipStream_t s, const char* what)
{
    hipError_t e = hipMemcpyAsync(c->h_pinned, c->scal, kSCount * sizeof(int), hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return hip_fail(c, e, what);
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(c, e, what);
    const int bits = c->h_pinned[kSErr];
    if (bits) {
        fill_i32(c->scal + kSErr, 1, 0, s);
        (void)hipStreamSynchronize(s);
        if (bits & kErrBitRange)
            return fail(c, GRAM_ERR_RANGE, "%s: an item ID outside [0, %d) was seen", what, c->cfg.vocab_n);
        return fail(c, GRAM_ERR_CAPACITY, "%s: the window touched more than %lld unique items", what,
                    (long long)c->cap_total);
    }
    return GRAM_OK;
}

}  // namespace

// ---- gram_unique for callers that cannot allocate -----------------------------------
//
// The dedup kernels need scratch memory (radix ping-pong arrays, digit tables, segment
// offsets).  gram_unique takes it from the context's workspace, which gram_create
// allocates; this variant takes it from one array in the library's device image, so it
// allocates nothing.  The array's name is a host-side stand-in, not a device address:
// its device address is looked up once per device and only that pointer is used below.
namespace {

constexpr int64_t kStaticMax = GRAM_UNIQUE_STATIC_MAX_POSITIONS;
constexpr int64_t static_align(int64_t v) { return (v + 255) / 256 * 256; }
// digit table of the largest sort plan (see table_elems_for): 256 blocks + 1, 1024 bins
constexpr int64_t kStaticTableElems = ((int64_t)1 << kMaxDigitBits) * 257;
constexpr int64_t kStaticOffScal = 0;
constexpr int64_t kStaticOffKeys0 = kStaticOffScal + static_align(64 * 4);
constexpr int64_t kStaticOffKeys1 = kStaticOffKeys0 + static_align(kStaticMax * 4);
constexpr int64_t kStaticOffVals0 = kStaticOffKeys1 + static_align(kStaticMax * 4);
constexpr int64_t kStaticOffVals1 = kStaticOffVals0 + static_align(kStaticMax * 4);
constexpr int64_t kStaticOffTable = kStaticOffVals1 + static_align(kStaticMax * 4);
constexpr int64_t kStaticOffGtot = kStaticOffTable + static_align(kStaticTableElems * 4);
constexpr int64_t kStaticOffTiles = kStaticOffGtot + static_align((1 << kMaxDigitBits) * 4);
constexpr int64_t kStaticOffOffsets = kStaticOffTiles + static_align((kStaticMax / kScanTile + 2) * 3 * 4);
constexpr int64_t kStaticOffSegOfRow = kStaticOffOffsets + static_align((kStaticMax + 2) * 4);
constexpr int64_t kStaticOffUniqWs = kStaticOffSegOfRow + static_align(kStaticMax * 4);
constexpr int64_t kStaticBytes = kStaticOffUniqWs + static_align(kStaticMax * 4);
static_assert(kStaticBytes < ((int64_t)9 << 20), "the static scratch array is meant to stay below 9 MiB");

constexpr int kStaticMaxDevices = 64;
std::mutex g_static_mutex;
unsigned char* g_static_ptr[kStaticMaxDevices] = {};

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

// Device address of `scratch` on the current device (looked up on the first call there).
int static_scratch(unsigned char** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(nullptr, e, "gram_unique_static: hipGetDevice");
    if (dev < 0 || dev >= kStaticMaxDevices)
        return fail(nullptr, GRAM_ERR_ARG, "gram_unique_static: device index %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(nullptr, e, "gram_unique_static: hipGetSymbolAddress");
        g_static_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_static_ptr[dev];
    return GRAM_OK;
}

__global__ void k_copy_scalar(const int* __restrict__ src, int* __restrict__ dst)
{
    if (threadIdx.x == 0) *dst = *src;
}

}  // namespace

extern "C" {

int64_t gram_workspace_bytes(const gram_config* cfg)
{
    Derived dv;
    if (validate(cfg, &dv)) return 0;
    return layout(nullptr, *cfg, dv, nullptr);
}

int gram_create(gram_ctx** out, const gram_config* cfg)
{
    if (!out) return fail(nullptr, GRAM_ERR_ARG, "gram_create: out is NULL");
    *out = nullptr;
    Derived dv;
    if (const char* why = validate(cfg, &dv)) return fail(nullptr, GRAM_ERR_ARG, "gram_create: %s", why);
    Ctx* c = new (std::nothrow) Ctx();
    if (!c) return fail(nullptr, GRAM_ERR_ARG, "gram_create: out of host memory");
    c->cfg = *cfg;
    c->cap_u = dv.cap_u;
    c->cap_total = dv.cap_total;
    c->cap_chunk = dv.cap_chunk;
    c->dense = cfg->buffer_layout == GRAM_BUFFER_DENSE;
    c->key_bits = bits_for(cfg->vocab_n);
    c->wg_splits = dv.splits;
    c->ws_bytes = layout(nullptr, *cfg, dv, nullptr);
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            c->num_cus = cus;
    }
    hipError_t e = hipMalloc((void**)&c->ws_base, (size_t)c->ws_bytes);
    if (e != hipSuccess) {
        int rc = fail(nullptr, GRAM_ERR_HIP, "gram_create: hipMalloc(%lld bytes): %s",
                      (long long)c->ws_bytes, hipGetErrorString(e));
        delete c;
        return rc;
    }
    layout(c, *cfg, dv, c->ws_base);
    e = hipHostMalloc((void**)&c->h_pinned, 64 * sizeof(int), hipHostMallocDefault);
    if (e != hipSuccess) {
        int rc = fail(nullptr, GRAM_ERR_HIP, "gram_create: hipHostMalloc: %s", hipGetErrorString(e));
        (void)hipFree(c->ws_base);
        delete c;
        return rc;
    }
    fill_i32(c->scal, 64, 0, nullptr);
    if (cfg->d_hidden > 0) iota_i32(c->iota, c->cap_chunk, nullptr);
    if (c->dense) {
        // rows and counts are zero outside a window; gram_flush restores that for what it exports
        fill_i32(reinterpret_cast<int*>(c->G), (int64_t)cfg->vocab_n * cfg->d, 0, nullptr);
        fill_i32(reinterpret_cast<int*>(c->cnt64), (int64_t)cfg->vocab_n * 2, 0, nullptr);
    } else {
        fill_i32(c->slot_of, cfg->vocab_n, -1, nullptr);
    }
    e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) {
        int rc = fail(nullptr, GRAM_ERR_HIP, "gram_create: init: %s", hipGetErrorString(e));
        (void)hipHostFree(c->h_pinned);
        (void)hipFree(c->ws_base);
        delete c;
        return rc;
    }
    *out = reinterpret_cast<gram_ctx*>(c);
    return GRAM_OK;
}

int gram_destroy(gram_ctx* ctx)
{
    if (!ctx) return GRAM_OK;
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    (void)hipDeviceSynchronize();
    for (ProfSlot& p : c->prof_pool) {
        (void)hipEventDestroy(p.start);
        (void)hipEventDestroy(p.stop);
    }
    if (c->h_pinned) (void)hipHostFree(c->h_pinned);
    if (c->ws_base) (void)hipFree(c->ws_base);
    delete c;
    return GRAM_OK;
}

int gram_unique(gram_ctx* ctx, const int32_t* ids, int64_t m, int32_t* uniq, int32_t* inverse,
                int32_t* counts, int32_t* u_dev, int32_t* u_host, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (m < 0) return fail(c, GRAM_ERR_ARG, "gram_unique: m < 0");
    if (m > c->cfg.max_positions)
        return fail(c, GRAM_ERR_CAPACITY, "gram_unique: m = %lld exceeds max_positions = %lld",
                    (long long)m, (long long)c->cfg.max_positions);
    if (m > 0 && (!ids || !uniq || !inverse || !counts))
        return fail(c, GRAM_ERR_ARG, "gram_unique: NULL pointer");
    hipStream_t s = static_cast<hipStream_t>(stream);
    c->have_unique = false;
    if (m > 0) {
        const int fix = c->cfg.pad_id >= 0 ? c->cfg.pad_id : 0;
        // slot-table contexts: the dedup kernels also work out the buffer rows of the items
        const bool prospect = !c->dense;
        const int first_step = (c->steps_done == 0 && !c->window_imported) ? 1 : 0;
        if (!unique_small(c, ids, (int)m, fix, uniq, inverse, counts, u_dev, s, prospect, first_step)) {
            const int r = radix_sort_pairs(c, ids, nullptr, (int)m, nullptr, m, true, fix, s);
            c->sorted_keys = c->keys[r];
            c->perm = c->vals[r];
            unique_from_sorted(c, (int)m, uniq, inverse, counts, u_dev, s, prospect, first_step);
        }
        c->prospect_epoch = prospect ? c->slot_epoch : 0;
    } else {
        unique_from_sorted(c, 0, uniq, inverse, counts, u_dev, s);
        c->prospect_epoch = 0;
    }
    if (int rc = launch_status(c, "gram_unique")) return rc;
    c->have_unique = true;
    c->last_uniq = uniq;
    c->last_inverse = inverse;
    c->unique_consumed = false;
    c->cur_m = m;
    if (u_host) {
        if (int rc = sync_scalars(c, s, "gram_unique")) return rc;
        *u_host = c->h_pinned[kSU];
    }
    return GRAM_OK;
}

int gram_encode_gather(gram_ctx* ctx, const void* X, const void* W, const int32_t* uniq,
                       const int32_t* inverse, const int32_t* u_dev, int64_t m, float* E, void* H,
                       void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (!c->have_unique)
        return fail(c, GRAM_ERR_SEQUENCE, "gram_encode_gather: no preceding gram_unique");
    if (m != c->cur_m)
        return fail(c, GRAM_ERR_ARG, "gram_encode_gather: m = %lld differs from the last gram_unique (%lld)",
                    (long long)m, (long long)c->cur_m);
    if (m > 0 && (!X || !W || !uniq || !inverse || !H))
        return fail(c, GRAM_ERR_ARG, "gram_encode_gather: NULL pointer");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (m == 0) return GRAM_OK;
    float* Ep = E ? E : c->E_ws;
    const int* up = u_dev ? u_dev : c->scal + kSU;
    // The fused epilogue walks the sorted order of the last dedup, so it applies only when the
    // caller hands back that call's own outputs.  It then takes the unique list from the context's
    // copy as well: rows and positions come from one and the same dedup, whatever the caller's
    // buffers hold by now.
    const bool own = uniq == c->last_uniq && inverse == c->last_inverse;
    if (encode_forward(c, X, W, own ? c->uniq_ws : uniq, own ? c->scal + kSU : up, m < c->cap_u ? m : c->cap_u, Ep,
                       s, own ? H : nullptr, E != nullptr))
        gather_heavy(c, Ep, m, H, s);
    else
        gather_rows(c, Ep, inverse, m, H, s);
    return launch_status(c, "gram_encode_gather");
}

int gram_mlp_encode_gather(gram_ctx* ctx, const void* X, const void* W1, const void* W2, const int32_t* uniq,
                           const int32_t* inverse, const int32_t* u_dev, int64_t m, void* A1, float* E,
                           void* H, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (c->cfg.d_hidden <= 0)
        return fail(c, GRAM_ERR_ARG, "gram_mlp_encode_gather: the context was created with d_hidden = 0");
    if (!c->have_unique)
        return fail(c, GRAM_ERR_SEQUENCE, "gram_mlp_encode_gather: no preceding gram_unique");
    if (m != c->cur_m)
        return fail(c, GRAM_ERR_ARG, "gram_mlp_encode_gather: m = %lld differs from the last gram_unique (%lld)",
                    (long long)m, (long long)c->cur_m);
    if (m > 0 && (!X || !W1 || !W2 || !uniq || !inverse || !H))
        return fail(c, GRAM_ERR_ARG, "gram_mlp_encode_gather: NULL pointer");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (m == 0) return GRAM_OK;
    float* Ep = E ? E : c->E_ws;
    const int* up = u_dev ? u_dev : c->scal + kSU;
    const bool own = uniq == c->last_uniq && inverse == c->last_inverse;
    if (mlp_forward(c, X, W1, W2, own ? c->uniq_ws : uniq, own ? c->scal + kSU : up, m < c->cap_u ? m : c->cap_u, A1,
                    Ep, s, own ? H : nullptr, E != nullptr))
        gather_heavy(c, Ep, m, H, s);
    else
        gather_rows(c, Ep, inverse, m, H, s);
    return launch_status(c, "gram_mlp_encode_gather");
}

int64_t gram_mlp_batch_bytes(const gram_ctx* ctx, int64_t n)
{
    const Ctx* c = reinterpret_cast<const Ctx*>(ctx);
    if (!c || c->cfg.d_hidden <= 0 || n < 0) return 0;
    return mlp_batch_bytes(c, n);
}

int gram_mlp_backward(gram_ctx* ctx, const void* X, const void* W1, const void* W2, const int32_t* ids,
                      const float* G_rows, const float* Ht, int64_t n, void* work, float* dW1, float* dW2,
                      int32_t accumulate, double* loss_dev, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (c->cfg.d_hidden <= 0)
        return fail(c, GRAM_ERR_ARG, "gram_mlp_backward: the context was created with d_hidden = 0");
    if (n < 0 || n > c->cap_chunk)
        return fail(c, GRAM_ERR_ARG, "gram_mlp_backward: n = %lld outside [0, %lld]", (long long)n,
                    (long long)c->cap_chunk);
    if ((G_rows != nullptr) == (Ht != nullptr) && n > 0)
        return fail(c, GRAM_ERR_ARG, "gram_mlp_backward: give exactly one of G_rows and Ht");
    if (!X || !W1 || !W2 || !dW1 || !dW2 || (n > 0 && (!ids || !work)))
        return fail(c, GRAM_ERR_ARG, "gram_mlp_backward: NULL pointer");
    mlp_backward(c, X, W1, W2, ids, G_rows, Ht, n, work, dW1, dW2, accumulate != 0, Ht ? loss_dev : nullptr,
                 static_cast<hipStream_t>(stream));
    return launch_status(c, "gram_mlp_backward");
}

int gram_grad_accumulate(gram_ctx* ctx, const float* dH, int64_t m, int32_t step_k, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (!c->have_unique || c->unique_consumed)
        return fail(c, GRAM_ERR_SEQUENCE, "gram_grad_accumulate: needs a fresh gram_unique for this batch");
    if (m != c->cur_m)
        return fail(c, GRAM_ERR_ARG, "gram_grad_accumulate: m = %lld differs from the last gram_unique (%lld)",
                    (long long)m, (long long)c->cur_m);
    if (step_k != c->steps_done || step_k >= c->cfg.k_steps)
        return fail(c, GRAM_ERR_SEQUENCE, "gram_grad_accumulate: step_k = %d, expected %d (k_steps = %d)",
                    step_k, c->steps_done, c->cfg.k_steps);
    if (m > 0 && !dH) return fail(c, GRAM_ERR_ARG, "gram_grad_accumulate: dH is NULL");
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the rows worked out by gram_unique hold if the slot table is still the one it looked at;
    // the reduction then commits them as it goes, else they are assigned afresh first
    const bool commit = m > 0 && c->prospect_epoch == c->slot_epoch;
    if (!commit) assign_slots(c, s);
    segment_reduce(c, dH, m, s, commit);
    c->slot_epoch += 1;
    if (int rc = launch_status(c, "gram_grad_accumulate")) return rc;
    c->unique_consumed = true;
    c->steps_done += 1;
    c->window_positions += m;
    return GRAM_OK;
}

int gram_pseudo_target(gram_ctx* ctx, const float* E, float* Ht, double* loss_dev, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (!c->have_unique || !c->unique_consumed)
        return fail(c, GRAM_ERR_SEQUENCE, "gram_pseudo_target: needs the gram_grad_accumulate of this batch");
    if (c->cur_m > 0 && (!E || (!Ht && !loss_dev)))
        return fail(c, GRAM_ERR_ARG, "gram_pseudo_target: E and at least one output are required");
    pseudo_target(c, E, Ht, loss_dev, static_cast<hipStream_t>(stream));
    return launch_status(c, "gram_pseudo_target");
}

int gram_gather(gram_ctx* ctx, const float* src, const int32_t* inverse, int64_t m, void* H, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (m < 0 || m > c->cfg.max_positions)
        return fail(c, GRAM_ERR_ARG, "gram_gather: m = %lld outside [0, max_positions]", (long long)m);
    if (m > 0 && (!src || !inverse || !H)) return fail(c, GRAM_ERR_ARG, "gram_gather: NULL pointer");
    gather_rows(c, src, inverse, m, H, static_cast<hipStream_t>(stream));
    return launch_status(c, "gram_gather");
}

int gram_encoder_wgrad(gram_ctx* ctx, const void* X, float* dW, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (c->steps_done < 1 && !c->window_imported)
        return fail(c, GRAM_ERR_SEQUENCE, "gram_encoder_wgrad: no step accumulated in this window");
    if (!X || !dW) return fail(c, GRAM_ERR_ARG, "gram_encoder_wgrad: NULL pointer");
    encoder_wgrad(c, X, dW, static_cast<hipStream_t>(stream), 0, c->cap_total, false);
    return launch_status(c, "gram_encoder_wgrad");
}

int gram_encoder_wgrad_chunk(gram_ctx* ctx, const void* X, float* dW, int64_t first_row, int64_t n_rows,
                             int32_t accumulate, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (c->steps_done < 1 && !c->window_imported)
        return fail(c, GRAM_ERR_SEQUENCE, "gram_encoder_wgrad_chunk: no step accumulated in this window");
    if (!X || !dW) return fail(c, GRAM_ERR_ARG, "gram_encoder_wgrad_chunk: NULL pointer");
    if (first_row < 0 || n_rows < 0)
        return fail(c, GRAM_ERR_ARG, "gram_encoder_wgrad_chunk: negative row range");
    encoder_wgrad(c, X, dW, static_cast<hipStream_t>(stream), first_row, n_rows, accumulate != 0);
    return launch_status(c, "gram_encoder_wgrad_chunk");
}

int gram_pseudo_loss_grad(gram_ctx* ctx, const void* X, const void* W, const int32_t* ids, const float* Ht,
                          int64_t n, float* R, float* dW, int32_t accumulate, double* loss_dev, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (n < 0 || n > c->cap_chunk)
        return fail(c, GRAM_ERR_ARG, "gram_pseudo_loss_grad: n = %lld outside [0, %lld]", (long long)n,
                    (long long)c->cap_chunk);
    if (!X || !W || !dW || (n > 0 && (!ids || !Ht || !R)))
        return fail(c, GRAM_ERR_ARG, "gram_pseudo_loss_grad: NULL pointer");
    hipStream_t s = static_cast<hipStream_t>(stream);
    chunk_ids_prepare(c, ids, n, s);
    if (c->cfg.xw_dtype == GRAM_BF16) {
        // the contraction subtracts the targets as it stores; only the loss needs another pass
        encode_forward(c, X, W, c->chunk_ids, c->scal + kSChunkN, n, R, s, nullptr, true, kEpiMinus, Ht);
        pseudo_miss(c, R, nullptr, n, loss_dev, s);
    } else {
        encode_forward(c, X, W, c->chunk_ids, c->scal + kSChunkN, n, R, s, nullptr, true);
        pseudo_miss(c, R, Ht, n, loss_dev, s);
    }
    const WgradRows rows = {c->chunk_ids, R, c->scal + kSChunkN, n};
    encoder_wgrad(c, X, dW, s, 0, n, accumulate != 0, &rows);
    return launch_status(c, "gram_pseudo_loss_grad");
}

static int flush_any(Ctx* c, int32_t* uniq_total, int32_t* counts_total, int64_t* counts64_total,
                     float* G_total, int32_t* u_total_dev, int32_t* u_total_host, hipStream_t s,
                     const char* what)
{
    if (c->dense)
        flush_dense(c, uniq_total, counts_total, reinterpret_cast<long long*>(counts64_total), G_total,
                    u_total_dev, s);
    else
        flush_export(c, uniq_total, counts_total, reinterpret_cast<long long*>(counts64_total), G_total,
                     u_total_dev, s);
    c->have_unique = false;     // the sort buffers were reused
    c->slot_epoch += 1;
    c->steps_done = 0;
    c->window_positions = 0;
    c->window_imported = false;
    if (int rc = launch_status(c, what)) return rc;
    if (u_total_host) {
        if (int rc = sync_scalars(c, s, what)) return rc;
        *u_total_host = c->h_pinned[kSFlushN];
    }
    return GRAM_OK;
}

int gram_flush(gram_ctx* ctx, int32_t* uniq_total, int32_t* counts_total, float* G_total,
               int32_t* u_total_dev, int32_t* u_total_host, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    return flush_any(c, uniq_total, counts_total, nullptr, G_total, u_total_dev, u_total_host,
                     static_cast<hipStream_t>(stream), "gram_flush");
}

int gram_flush64(gram_ctx* ctx, int32_t* uniq_total, int64_t* counts_total, float* G_total,
                 int32_t* u_total_dev, int32_t* u_total_host, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    return flush_any(c, uniq_total, nullptr, counts_total, G_total, u_total_dev, u_total_host,
                     static_cast<hipStream_t>(stream), "gram_flush64");
}

int gram_window_end(gram_ctx* ctx, const void* X, float* dW, int32_t* uniq_total, int32_t* counts_total,
                    float* G_total, int32_t* u_total_dev, int32_t* u_total_host, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (c->steps_done < 1 && !c->window_imported)
        return fail(c, GRAM_ERR_SEQUENCE, "gram_window_end: no step accumulated in this window");
    if (!X || !dW) return fail(c, GRAM_ERR_ARG, "gram_window_end: NULL pointer");
    hipStream_t s = static_cast<hipStream_t>(stream);
    // The fused form: the weight-gradient kernel holds every buffer row in registers on its way
    // into LDS and writes it to its place in the export from there, so the rows are read once.
    const bool fused = !c->dense && G_total && c->cfg.xw_dtype == GRAM_BF16 &&
                       (int64_t)c->cfg.vocab_n * c->cfg.d_in * 2 < kBufferWindow &&
                       c->cap_total * (int64_t)c->cfg.d * 4 < kBufferWindow;
    if (!fused) {
        encoder_wgrad(c, X, dW, s, 0, c->cap_total, false);
        return flush_any(c, uniq_total, counts_total, nullptr, G_total, u_total_dev, u_total_host, s,
                         "gram_window_end");
    }
    bool meta_left = false;
    const int* ranks = flush_meta_and_ranks(c, uniq_total, counts_total, u_total_dev, s, &meta_left);
    const WindowMeta meta = {uniq_total, counts_total, u_total_dev};
    encoder_wgrad(c, X, dW, s, 0, c->cap_total, false, nullptr, G_total, ranks, meta_left ? &meta : nullptr);
    c->have_unique = false;     // the sort buffers were reused
    c->slot_epoch += 1;
    c->steps_done = 0;
    c->window_positions = 0;
    c->window_imported = false;
    if (int rc = launch_status(c, "gram_window_end")) return rc;
    if (u_total_host) {
        if (int rc = sync_scalars(c, s, "gram_window_end")) return rc;
        *u_total_host = c->h_pinned[kSFlushN];
    }
    return GRAM_OK;
}

int gram_window_import(gram_ctx* ctx, const int32_t* ids, const int64_t* counts, const float* G_rows,
                       int64_t n, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    const int64_t n_max = c->dense ? c->cfg.vocab_n : c->cap_total;
    if (n < 0 || n > n_max)
        return fail(c, GRAM_ERR_ARG, "gram_window_import: n = %lld outside [0, %lld]", (long long)n,
                    (long long)n_max);
    if (n > 0 && (!ids || !counts)) return fail(c, GRAM_ERR_ARG, "gram_window_import: NULL pointer");
    if (c->dense)
        import_dense(c, ids, reinterpret_cast<const long long*>(counts), G_rows, n, static_cast<hipStream_t>(stream));
    else
        import_slots(c, ids, reinterpret_cast<const long long*>(counts), G_rows, n, static_cast<hipStream_t>(stream));
    c->slot_epoch += 1;
    if (int rc = launch_status(c, "gram_window_import")) return rc;
    c->window_imported = true;
    c->window_positions += n;      // host bound on the rows in the buffer (sizes the split-K of the weight gradient)
    return GRAM_OK;
}

static const char* const kKernelNames[KID_COUNT] = {
    "radix_hist", "radix_scan", "radix_scatter", "heads_count", "heads_emit", "unique_empty",
    "transpose_w", "encode_bf16", "encode_f32", "gather_rows", "slot_count", "slot_emit", "seg_reduce",
    "seg_combine", "wgrad_bf16", "wgrad_f32", "wgrad_reduce", "flush_meta",
    "flush_rows", "unique_small", "gather_heavy", "pseudo_target", "pseudo_loss", "chunk_ids",
    "pseudo_miss", "mlp_to_bf16", "encode_bf16_wide", "wgrad_bf16_wide"};

int gram_kernel_count(void) { return KID_COUNT; }

int gram_light_max(void) { return kLightMax; }

const char* gram_kernel_name(int k) { return (k >= 0 && k < KID_COUNT) ? kKernelNames[k] : ""; }

int gram_profile_enable(gram_ctx* ctx, uint64_t mask, int32_t max_launches)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    if (max_launches < 0 || max_launches > (1 << 20))
        return fail(c, GRAM_ERR_ARG, "gram_profile_enable: max_launches out of range");
    (void)hipDeviceSynchronize();
    while (c->prof_pool.size() < (size_t)max_launches) {
        ProfSlot p{};
        hipError_t e = hipEventCreate(&p.start);
        if (e == hipSuccess) e = hipEventCreate(&p.stop);
        if (e != hipSuccess) return hip_fail(c, e, "gram_profile_enable");
        c->prof_pool.push_back(p);
    }
    c->prof_used = 0;
    c->prof_mask = mask;
    return GRAM_OK;
}

int gram_profile_read(gram_ctx* ctx, int k, int64_t* launches, double* total_ms)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c || !launches || !total_ms || k < 0 || k >= KID_COUNT) return GRAM_ERR_ARG;
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return hip_fail(c, e, "gram_profile_read");
    int64_t n = 0;
    double ms = 0.0;
    for (size_t i = 0; i < c->prof_used; ++i) {
        const ProfSlot& p = c->prof_pool[i];
        if (p.kid != k) continue;
        float t = 0.f;
        e = hipEventElapsedTime(&t, p.start, p.stop);
        if (e != hipSuccess) return hip_fail(c, e, "gram_profile_read");
        ms += t;
        ++n;
    }
    *launches = n;
    *total_ms = ms;
    return GRAM_OK;
}

int gram_unique_static(const int32_t* ids, int64_t m, int32_t vocab_n, int32_t pad_id, int32_t* uniq,
                       int32_t* inverse, int32_t* counts, int32_t* u_dev, int32_t* err_dev, void* stream)
{
    if (m < 0) return fail(nullptr, GRAM_ERR_ARG, "gram_unique_static: m < 0");
    if (m > kStaticMax)
        return fail(nullptr, GRAM_ERR_CAPACITY, "gram_unique_static: m = %lld exceeds the fixed maximum of %lld positions",
                    (long long)m, (long long)kStaticMax);
    if (vocab_n < 1 || pad_id >= vocab_n)
        return fail(nullptr, GRAM_ERR_ARG, "gram_unique_static: vocab_n must be >= 1 and pad_id < vocab_n");
    if (!u_dev || (m > 0 && (!ids || !uniq || !inverse || !counts)))
        return fail(nullptr, GRAM_ERR_ARG, "gram_unique_static: NULL pointer");
    unsigned char* base = nullptr;
    if (int rc = static_scratch(&base)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);

    // A context on the stack whose workspace pointers lie in the static array: the kernels are
    // the ones gram_unique runs.
    Ctx c;
    c.cfg = gram_config{};
    c.cfg.vocab_n = vocab_n;
    c.cfg.pad_id = pad_id;
    c.cfg.max_positions = kStaticMax;
    c.cap_u = kStaticMax < vocab_n ? kStaticMax : vocab_n;
    c.key_bits = bits_for(vocab_n);
    c.scal = reinterpret_cast<int*>(base + kStaticOffScal);
    c.keys[0] = reinterpret_cast<int*>(base + kStaticOffKeys0);
    c.keys[1] = reinterpret_cast<int*>(base + kStaticOffKeys1);
    c.vals[0] = reinterpret_cast<int*>(base + kStaticOffVals0);
    c.vals[1] = reinterpret_cast<int*>(base + kStaticOffVals1);
    c.table = reinterpret_cast<int*>(base + kStaticOffTable);
    c.gtot = reinterpret_cast<int*>(base + kStaticOffGtot);
    c.tile_sums = reinterpret_cast<int*>(base + kStaticOffTiles);
    c.offsets = reinterpret_cast<int*>(base + kStaticOffOffsets);
    c.seg_of_row = reinterpret_cast<int*>(base + kStaticOffSegOfRow);
    c.uniq_ws = reinterpret_cast<int*>(base + kStaticOffUniqWs);

    // the array keeps the last call's contents: the error bits must start at zero (a fill kernel,
    // so that the call can be captured in a HIP graph); everything else is written before it is read
    fill_i32(c.scal, 64, 0, s);
    if (m > 0) {
        const int fix = pad_id >= 0 ? pad_id : 0;
        if (!unique_small(&c, ids, (int)m, fix, uniq, inverse, counts, u_dev, s)) {
            const int r = radix_sort_pairs(&c, ids, nullptr, (int)m, nullptr, m, true, fix, s);
            c.sorted_keys = c.keys[r];
            c.perm = c.vals[r];
            unique_from_sorted(&c, (int)m, uniq, inverse, counts, u_dev, s);
        }
    } else {
        unique_from_sorted(&c, 0, uniq, inverse, counts, u_dev, s);
    }
    if (err_dev) hipLaunchKernelGGL(k_copy_scalar, dim3(1), dim3(kWave), 0, s, c.scal + kSErr, err_dev);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(nullptr, e, "gram_unique_static");
    return GRAM_OK;
}

int gram_check(gram_ctx* ctx, void* stream)
{
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (!c) return GRAM_ERR_ARG;
    return sync_scalars(c, static_cast<hipStream_t>(stream), "gram_check");
}

const char* gram_last_error(const gram_ctx* ctx)
{
    const Ctx* c = reinterpret_cast<const Ctx*>(ctx);
    return c ? c->last_error.c_str() : g_create_error.c_str();
}

}  // extern "C"
