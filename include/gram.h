/*
 * gram.h -- C ABI of the MI355X (gfx950) library for GRAM's data-parallel hot
 * path: the item-deduplicated encode / gradient-accumulate step of
 * content-based collaborative filtering (Section 4, Algorithm 1 of the paper).
 *
 * One training step over a mini-batch of M = B*L item-ID positions:
 *
 *   gram_unique           the set B_I of unique items of the batch (Table 1;
 *                         "for all i in B_I" in Algorithm 1), ascending, with
 *                         the inverse index and multiplicities
 *   gram_encode_gather    step 1, Eq. 4: one representation per unique item
 *                         (dense linear stand-in for the encoder, E = X[uniq].W),
 *                         gathered back to every position
 *   gram_grad_accumulate  step 3, Eq. 6: dL/dH summed per unique item into the
 *                         buffer that persists over the N mini-batches of a
 *                         Multi-step window (Section 4.2)
 *   gram_pseudo_target    step 3 as the paper writes it: the pseudo-target
 *                         h~ = h - grad L(h) of each item of the batch and the
 *                         pseudo-loss of Eq. 7 (optional; gram_gather gathers
 *                         such rows to positions)
 *   gram_encoder_wgrad    step 4, Eq. 7/9: encoder weight gradient once per
 *                         unique item, dW = X[items]^T . G
 *   gram_flush            end of the window ("t mod N"): export and empty the
 *                         buffer
 *   gram_pseudo_loss_grad step 4 as a regression towards stored pseudo-targets,
 *                         one content-encoder batch at a time, at the encoder's
 *                         current weights (optional)
 *   gram_encoder_wgrad_chunk  the weight gradient over a range of the window's
 *                         items (content-encoder batches; optional)
 *   gram_window_end       gram_encoder_wgrad + gram_flush reading the buffer once
 *   gram_flush64, gram_window_import   64-bit counts and save / resume of a
 *                         window kept in the dense one-row-per-ID buffer
 *                         (cfg.buffer_layout; windows of epoch length)
 *   gram_mlp_encode_gather, gram_mlp_backward   steps 1 and 4 with a two-layer
 *                         stand-in encoder (cfg.d_hidden > 0)
 *
 * Memory.  Every pointer marked DEVICE is memory of the current HIP device,
 * owned by the caller (the library never frees, reallocates or keeps it beyond
 * the call unless stated).  Pointers marked HOST are ordinary host memory.
 * gram_create allocates all workspace once; no later call allocates.
 *
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = default
 * stream).  Calls only enqueue work; they synchronise with the host only where
 * a HOST out-pointer is non-NULL, and in gram_check.  One context serves one
 * stream at a time and is not re-entrant.
 *
 * Layouts.  All matrices are dense row-major.  ids/uniq/inverse/counts are
 * int32.  X[N,d_in] and W[d_in,d] have the context's xw_dtype; E, H, dH, G and
 * dW are float32 (the paper does not state a precision; sums are taken in
 * float32 in a fixed order, so results are bit-reproducible run to run).
 *
 * Errors.  Functions return GRAM_OK (0) or a negative gram_status and leave a
 * message for gram_last_error.  Errors the device detects (an ID outside
 * [0,N), buffer capacity exceeded) are latched in a device flag and returned
 * by the next call that synchronises (a HOST out-pointer, or gram_check);
 * an out-of-range ID is processed as the padding ID (0 if there is none) so no
 * kernel reads out of bounds, and the outputs of that step are unspecified.
 */
#ifndef GRAM_H
#define GRAM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gram_ctx gram_ctx; /* opaque: workspace + persistent gradient buffer */

typedef enum gram_status {
    GRAM_OK = 0,
    GRAM_ERR_ARG = -1,           /* NULL / negative / unsupported argument            */
    GRAM_ERR_CAPACITY = -2,      /* m > max_positions, or the window touched more
                                    unique items than u_total_cap                     */
    GRAM_ERR_SEQUENCE = -3,      /* call order violated (see each function)           */
    GRAM_ERR_RANGE = -4,         /* an ID outside [0, vocab_n)                        */
    GRAM_ERR_HIP = -5,           /* HIP runtime error; text in gram_last_error        */
    GRAM_ERR_UNIMPLEMENTED = -6
} gram_status;

typedef enum gram_dtype { GRAM_F32 = 0, GRAM_BF16 = 1 } gram_dtype;

/* Layout of the persistent gradient buffer.
 * GRAM_BUFFER_SLOTS: a compact table; an item gets the next free row when the
 *   window first meets it.  Sized for min(K*M_max, N) items (or u_total_cap).
 * GRAM_BUFFER_DENSE: one row per ID, G[N,d], like an embedding matrix; no slot
 *   map, counts are kept in 64 bits.  Meant for windows of epoch length
 *   (Section 4.2 and the half-epoch / one-epoch alternation periods of the
 *   experiments), where the window reaches most of the vocabulary: the weight
 *   gradient then contracts over all N rows (rows of items the window has not
 *   met are zero). */
typedef enum gram_buffer_layout { GRAM_BUFFER_SLOTS = 0, GRAM_BUFFER_DENSE = 1 } gram_buffer_layout;

typedef struct gram_config {
    int32_t vocab_n;       /* N: IDs are valid in [0,N); row r of X belongs to ID r    */
    int32_t d_in;          /* content-feature width; multiple of 8                     */
    int32_t d;             /* representation width; multiple of 4                      */
    int64_t max_positions; /* capacity M_max = B*L of one step                         */
    int32_t k_steps;       /* N of Algorithm 1 (accumulation period), >= 1             */
    int32_t pad_id;        /* padding ID (0 in the paper-shaped workloads); < 0: none  */
    int64_t u_total_cap;   /* rows of the persistent buffer; 0 => min(K*M_max, N)      */
    int32_t xw_dtype;      /* gram_dtype of X and W                                    */
    int32_t buffer_layout; /* gram_buffer_layout; DENSE: u_total_cap must be 0 or N    */
    int32_t d_hidden;      /* 0: linear stand-in encoder.  > 0: width of the hidden
                              layer of the two-layer stand-in (gram_mlp_*; bf16 only,
                              d_hidden and d multiples of 8)                           */
    int32_t h_dtype;       /* gram_dtype of H, the per-position output of the forward:
                              GRAM_F32 (0), or GRAM_BF16: each value is rounded to
                              nearest even as it is stored (half the bytes of the
                              step's largest output); E stays float32                  */
} gram_config;

/* Bytes of device memory gram_create would allocate for cfg (0 if cfg is invalid). */
int64_t gram_workspace_bytes(const gram_config* cfg);

/* Create a context on the current device.  Allocates the workspace and the
 * persistent buffer (hipMalloc) and initialises them on the default stream,
 * then synchronises.  *out is NULL on failure. */
int gram_create(gram_ctx** out, const gram_config* cfg);

/* Frees everything gram_create allocated.  Synchronises the device first. */
int gram_destroy(gram_ctx* ctx);

/* Unique items of a batch (Table 1, B_I; Eq. 4 ranges over it).
 *   ids      DEVICE [m]            item IDs, row-major [B,L]; padding = cfg.pad_id
 *   m        0 <= m <= max_positions
 *   uniq     DEVICE [>= min(m,N)]  out: distinct IDs ascending (padding included
 *                                  when present); entries >= U untouched
 *   inverse  DEVICE [m]            out: uniq[inverse[p]] == ids[p]
 *   counts   DEVICE [>= min(m,N)]  out: occurrences of uniq[j]; sums to m
 *   u_dev    DEVICE [1], nullable  out: U
 *   u_host   HOST   [1], nullable  out: U; non-NULL makes the call synchronise
 *                                  and return latched device errors
 * The context keeps the sort order of this batch for the next
 * gram_encode_gather / gram_grad_accumulate; a new gram_unique replaces it. */
int gram_unique(gram_ctx* ctx, const int32_t* ids, int64_t m, int32_t* uniq, int32_t* inverse,
                int32_t* counts, int32_t* u_dev, int32_t* u_host, void* stream);

/* Encode once per unique item and gather to positions (Algorithm 1 step 1).
 *   X        DEVICE [N,d_in]   item content features (xw_dtype)
 *   W        DEVICE [d_in,d]   encoder weight (xw_dtype)
 *   uniq, inverse, u_dev       the outputs of the preceding gram_unique (DEVICE)
 *   m        the m of that gram_unique
 *   E        DEVICE [>= min(m,N), d], nullable   out: E[j,:] = X[uniq[j],:].W,
 *            zero row for the padding ID; NULL keeps E in the workspace
 *   H        DEVICE [m,d] of cfg.h_dtype   out: H[p,:] = E[inverse[p],:] (zero at
 *            padding), rounded to nearest even when h_dtype is bf16; 16-byte aligned
 * Requires a preceding gram_unique on this context (GRAM_ERR_SEQUENCE); uniq and
 * inverse must hold what that call wrote, unmodified.
 * When uniq and inverse are the very buffers that gram_unique wrote (same
 * addresses), large bf16 batches take a fused path: the contraction stores each
 * representation straight to the positions of its item and E is written only if
 * the caller passes a buffer for it; an item with more than gram_light_max()
 * positions is copied to them by a second kernel.  That path reads the unique
 * list and the sort order from the context's own copies, not from the caller's
 * buffers, so rows and positions always belong to the same dedup (the batch of
 * the preceding gram_unique).  Any other uniq / inverse pair takes the
 * two-kernel path (encode to E, then gather), which reads the caller's buffers.
 * For unmodified buffers the results are identical. */
int gram_encode_gather(gram_ctx* ctx, const void* X, const void* W, const int32_t* uniq,
                       const int32_t* inverse, const int32_t* u_dev, int64_t m, float* E, void* H,
                       void* stream);

/* Per-unique-item gradient (Algorithm 1 step 3): for the batch of the last
 * gram_unique, G[item] += sum over the item's positions p (ascending) of
 * dH[p,:], into the persistent buffer.  Padding positions are not read.
 *   dH       DEVICE [m,d]  upstream gradient dL/dH
 *   m        must equal the m of the last gram_unique
 *   step_k   0-based step of the window; must equal the number of steps
 *            accumulated since the last gram_flush and be < k_steps
 * No float atomics are used: every buffer row has one writer and a fixed
 * summation order. */
int gram_grad_accumulate(gram_ctx* ctx, const float* dH, int64_t m, int32_t step_k, void* stream);

/* ---- A deeper stand-in encoder -----------------------------------------------
 * Eq. 4 takes any content encoder and the Proposition (Eq. 1-3) holds for any f.
 * With cfg.d_hidden > 0 the context also offers a two-layer encoder
 *   z = x . W1      a = max(z, 0)      h = a . W2,     W1 [d_in, d_hidden], W2 [d_hidden, d]
 * so that what the paper's section on GPU memory consumption is about can be
 * measured: the activation a, which the backward pass needs, is kept once per
 * unique item (bf16) instead of once per interaction.  gram_unique,
 * gram_grad_accumulate, gram_pseudo_target, gram_gather and gram_flush are used as
 * with the linear encoder; the two calls below replace gram_encode_gather and the
 * weight-gradient calls.  bf16 features and weights only.
 *
 * gram_mlp_encode_gather: Algorithm 1 step 1 with the two-layer encoder.
 *   W1, W2   DEVICE bf16       A1  DEVICE [>= U, d_hidden] bf16, nullable  out: the
 *                              hidden activations of the unique items (zero row for
 *                              the padding ID); other arguments as gram_encode_gather
 * gram_mlp_batch_bytes: bytes of `work` that gram_mlp_backward needs for n items
 *   (n * (6 d_hidden + 6 d), each of four parts rounded up to 256 bytes).
 * gram_mlp_backward: Algorithm 1 step 4 for one content-encoder batch of items.
 *   The activations are recomputed from the CURRENT weights (W1), so the call
 *   keeps nothing between batches but the caller's `work`.  Exactly one of
 *     G_rows  DEVICE [n,d]  dL/dh of each listed item (rows of gram_flush's
 *                           G_total: by the Proposition the result is the
 *                           end-to-end gradient when the weights have not moved)
 *     Ht      DEVICE [n,d]  stored pseudo-targets: the miss h - Ht at the current
 *                           weights is back-propagated and loss_dev (nullable)
 *                           receives the pseudo-loss of Eq. 7
 *   is given.  dW2 (+)= sum_j a_j^T r_j;  dz_j = (r_j . W2^T) where a_j > 0;
 *   dW1 (+)= sum_j X[ids[j],:]^T dz_j.  r and dz are rounded to bf16 as they enter
 *   the matrix cores.
 *   ids      DEVICE [n] int32 (range-checked like gram_pseudo_loss_grad's)
 *   n        0 <= n <= max(min(max_positions, N), rows of the buffer)
 *   work     DEVICE, gram_mlp_batch_bytes(ctx, n) bytes, 256-byte aligned
 *   dW1      DEVICE [d_in, d_hidden]   dW2  DEVICE [d_hidden, d]   float32 out;
 *            accumulate = 0 overwrites both, else adds */
int gram_mlp_encode_gather(gram_ctx* ctx, const void* X, const void* W1, const void* W2,
                           const int32_t* uniq, const int32_t* inverse, const int32_t* u_dev, int64_t m,
                           void* A1, float* E, void* H, void* stream);
int64_t gram_mlp_batch_bytes(const gram_ctx* ctx, int64_t n);
int gram_mlp_backward(gram_ctx* ctx, const void* X, const void* W1, const void* W2, const int32_t* ids,
                      const float* G_rows, const float* Ht, int64_t n, void* work, float* dW1,
                      float* dW2, int32_t accumulate, double* loss_dev, void* stream);

/* Pseudo-targets of the items of the current batch (Algorithm 1 step 3, Eq. 6:
 * the representation is moved by one plain gradient step of rate 1, Section 4.3)
 * and the pseudo-loss of Eq. 7 at the current encoder.
 *   E        DEVICE [>= U, d]   the representations gram_encode_gather wrote for
 *                               this batch (pass it a buffer for E)
 *   Ht       DEVICE [>= U, d], nullable   out: Ht[j,:] = E[j,:] - G(uniq[j]),
 *            G = the gradient accumulated for the item so far in the window,
 *            this batch included; zero row for the padding ID
 *   loss_dev DEVICE [1] double, nullable  out: 1/2 sum_j |Ht[j,:] - E[j,:]|^2
 *            (summed in double in a fixed order)
 * Requires the gram_grad_accumulate of this batch (GRAM_ERR_SEQUENCE); rows
 * >= U are untouched.  16-byte aligned pointers. */
int gram_pseudo_target(gram_ctx* ctx, const float* E, float* Ht, double* loss_dev, void* stream);

/* The gather step alone: H[p,:] = src[inverse[p],:] for p < m, e.g. to feed the
 * collaborative-filtering model with pseudo-targets instead of fresh
 * representations in later steps of a window (Section 4.3: item vectors as
 * trainable embeddings).
 *   src      DEVICE [>= U, d]   inverse  DEVICE [m], values < U
 *   H        DEVICE [m, d] of cfg.h_dtype      16-byte aligned pointers */
int gram_gather(gram_ctx* ctx, const float* src, const int32_t* inverse, int64_t m, void* H,
                void* stream);

/* Encoder weight gradient over all items accumulated in the window
 * (Algorithm 1 step 4): dW[i,c] = sum_items X[item,i] * G[item,c].
 *   X        DEVICE [N,d_in]
 *   dW       DEVICE [d_in,d]  out (overwritten)
 * Requires at least one accumulated step (GRAM_ERR_SEQUENCE).  Call before
 * gram_flush.  With bf16 features G is rounded to bf16 (nearest-even) as it
 * enters the matrix cores; products are summed in float32. */
int gram_encoder_wgrad(gram_ctx* ctx, const void* X, float* dW, void* stream);

/* The same weight gradient over a chunk of the accumulated items, for an encoder
 * update that walks the items of the window in batches of a fixed size (the
 * content-encoder batch size of the paper's section on GPU memory consumption
 * and its table):
 *   dW (+)= sum over buffer rows s in [first_row, first_row + n_rows) of
 *           X[item_s,:]^T . G[s,:]
 *   first_row, n_rows  rows of the buffer in the order the items entered the
 *                      window (ascending ID within a step, step after step); the
 *                      range is clipped to the rows held
 *   accumulate         0: dW is overwritten; otherwise the chunk is added to dW
 * The chunks of a partition of the held rows add up to gram_encoder_wgrad's dW
 * (up to the order of the float32 sums).  No workspace grows with the chunk.
 * With the dense buffer the rows are the IDs themselves: the chunk is the ID
 * range [first_row, first_row + n_rows). */
int gram_encoder_wgrad_chunk(gram_ctx* ctx, const void* X, float* dW, int64_t first_row,
                             int64_t n_rows, int32_t accumulate, void* stream);

/* One content-encoder batch of the update of Algorithm 1 step 4, written as the
 * paper states it: the encoder is regressed towards the pseudo-targets of the
 * listed items (pseudo-loss of Eq. 7), at the weights it has NOW, which may have
 * moved since the targets were taken (an optimiser step per batch; the
 * content-encoder batch size of the section on GPU memory consumption):
 *   h_j   = X[ids[j],:] . W
 *   R[j,:] = h_j - Ht[j,:]             (zero row for the padding ID)
 *   loss  = 1/2 sum_j |Ht[j,:] - h_j|^2
 *   dW (+)= sum_j X[ids[j],:]^T . R[j,:]
 * With targets taken at the same W this is gram_encoder_wgrad's gradient over
 * those items (Proposition, Eq. 1-3).
 *   X        DEVICE [N,d_in]    W  DEVICE [d_in,d]   (the context's xw_dtype)
 *   ids      DEVICE [n] int32   items of the batch, e.g. a range of gram_flush's
 *                               uniq_total; an ID outside [0,N) latches
 *                               GRAM_ERR_RANGE (reported by the next call that
 *                               synchronises) and counts as the padding item
 *   Ht       DEVICE [n,d]       their pseudo-targets
 *   n        0 <= n <= max(min(max_positions, N), rows of the buffer)
 *   R        DEVICE [n,d]       out: the regression miss; also the only workspace
 *                               the call needs beyond the context's
 *   dW       DEVICE [d_in,d]    out; accumulate = 0 overwrites, else adds
 *   loss_dev DEVICE [1] double, nullable  out (summed in double, fixed order)
 * With bf16 features R is rounded to bf16 (nearest-even) as it enters the matrix
 * cores, like G in gram_encoder_wgrad.  Independent of the window's state: may
 * be called at any point.  16-byte aligned pointers. */
int gram_pseudo_loss_grad(gram_ctx* ctx, const void* X, const void* W, const int32_t* ids,
                          const float* Ht, int64_t n, float* R, float* dW, int32_t accumulate,
                          double* loss_dev, void* stream);

/* End of the accumulation window: export the buffer in ascending ID order,
 * then empty it and reset the step counter.
 *   uniq_total    DEVICE [>= u_total_cap], nullable  out: IDs seen in the window
 *   counts_total  DEVICE [>= u_total_cap], nullable  out: their total occurrences
 *   G_total       DEVICE [>= u_total_cap, d], nullable  out: their gradient rows
 *   u_total_dev   DEVICE [1], nullable  out: number of IDs exported
 *   u_total_host  HOST   [1], nullable  out: same; non-NULL synchronises and
 *                                       returns latched device errors */
int gram_flush(gram_ctx* ctx, int32_t* uniq_total, int32_t* counts_total, float* G_total,
               int32_t* u_total_dev, int32_t* u_total_host, void* stream);

/* gram_flush with the counts in 64 bits.  Both buffer layouts keep 64-bit counts
 * (an epoch-long window can meet one item, the padding item above all, more
 * than 2^31 times; gram_flush itself saturates such a count at INT32_MAX).  Same
 * arguments otherwise; with the dense buffer the outputs need room for N items. */
int gram_flush64(gram_ctx* ctx, int32_t* uniq_total, int64_t* counts_total, float* G_total,
                 int32_t* u_total_dev, int32_t* u_total_host, void* stream);

/* gram_encoder_wgrad followed by gram_flush as one call, for the end of a window
 * (Algorithm 1 step 4 and the "t mod N" reset after it): same arguments, same
 * outputs as the two calls in that order.  With the slot-table buffer, bf16
 * features and operands below 4 GiB the weight-gradient kernel writes each buffer
 * row to its place in G_total while it holds the row for the contraction, so the
 * buffer is read once instead of twice; G_total then holds the same float32 rows
 * as gram_flush would write, and dW the same sums in the same order.  Otherwise
 * the call runs the two steps one after the other.
 *   X, dW          as for gram_encoder_wgrad
 *   uniq_total, counts_total, G_total, u_total_dev, u_total_host
 *                  as for gram_flush
 * Requires at least one accumulated step (GRAM_ERR_SEQUENCE). */
int gram_window_end(gram_ctx* ctx, const void* X, float* dW, int32_t* uniq_total,
                    int32_t* counts_total, float* G_total, int32_t* u_total_dev,
                    int32_t* u_total_host, void* stream);

/* Merge a saved window state into the buffer, e.g. what gram_flush64 exported
 * before an interruption: counts[j] is added to the count of ids[j] and, if
 * given, G_rows[j,:] to its gradient row.  A window saved after some
 * steps, imported and continued ends like the uninterrupted window (Section
 * 4.2: the buffer is the whole state of a window).
 *   ids     DEVICE [n] int32    distinct IDs (any order); an ID outside [0,N)
 *                               latches GRAM_ERR_RANGE and is skipped
 *   counts  DEVICE [n] int64    G_rows  DEVICE [n,d], nullable
 *   n       at most the rows of the buffer (N for the dense layout)
 * Does not count as a step (the next gram_grad_accumulate keeps its index) but
 * makes the window non-empty for gram_encoder_wgrad.  Slot table: items the
 * window has not met take rows in list order (GRAM_ERR_CAPACITY latched when
 * the buffer is full).  Uses the workspace of the
 * content-encoder batch calls (gram_pseudo_loss_grad, gram_mlp_backward). */
int gram_window_import(gram_ctx* ctx, const int32_t* ids, const int64_t* counts, const float* G_rows,
                       int64_t n, void* stream);

/* gram_unique for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Needs no
 * context: the scratch memory of the dedup kernels (sort buffers, digit tables,
 * segment offsets; about 8.3 MB) is one array in the library's device image, which
 * every GPU the library runs on holds until the process ends.  The call allocates
 * nothing and never synchronises; it only enqueues kernels on `stream`.
 *   ids, uniq, inverse, counts   DEVICE, as for gram_unique (uniq and counts with
 *                                room for min(m, vocab_n) entries)
 *   m        0 <= m <= GRAM_UNIQUE_STATIC_MAX_POSITIONS, else GRAM_ERR_CAPACITY
 *   vocab_n  IDs are valid in [0, vocab_n)       pad_id  as gram_config.pad_id
 *   u_dev    DEVICE [1]            out: U (required: there is no host copy)
 *   err_dev  DEVICE [1], nullable  out: 0, or 1 if an ID outside [0, vocab_n) was
 *                                  seen (such an ID is processed as the padding ID,
 *                                  0 if there is none)
 * Results are those of gram_unique, bit for bit.  All calls on one GPU share the
 * one array, which keeps the last call's contents (the call clears what must start
 * at zero itself): calls that overlap on one GPU, on different streams or host
 * threads, race.  Errors are reported through the return value and
 * gram_last_error(NULL). */
#define GRAM_UNIQUE_STATIC_MAX_POSITIONS 262144
int gram_unique_static(const int32_t* ids, int64_t m, int32_t vocab_n, int32_t pad_id, int32_t* uniq,
                       int32_t* inverse, int32_t* counts, int32_t* u_dev, int32_t* err_dev, void* stream);

/* Synchronise `stream` and return (and clear) any latched device error. */
int gram_check(gram_ctx* ctx, void* stream);

/* ---- Measurement aid (not a step of the paper's method) -------------------
 * The library can bracket its own kernel launches with HIP events on the
 * caller's stream, so a benchmark can report per-kernel durations without an
 * external profiler.  Kernel indices run over [0, gram_kernel_count()).
 *   gram_profile_enable  mask bit k set = time kernel k; 0 switches timing off.
 *                        The first call creates a fixed pool of events
 *                        (`max_launches` pairs, not in the hot path); launches
 *                        beyond the pool are not timed.  Discards earlier
 *                        readings.
 *   gram_profile_read    synchronises the device, then returns, for kernel k,
 *                        the number of timed launches and their summed duration
 *                        in milliseconds (HOST out-pointers).  Does not reset.
 */
int gram_kernel_count(void);
const char* gram_kernel_name(int k);
/* Largest number of positions of an item that the fused forward still stores
 * from the contraction's epilogue (a benchmark needs it to count the bytes
 * each of the two forward kernels moves). */
int gram_light_max(void);
int gram_profile_enable(gram_ctx* ctx, uint64_t mask, int32_t max_launches);
int gram_profile_read(gram_ctx* ctx, int k, int64_t* launches, double* total_ms);

/* Message of the last failing call on ctx (or of the last failing gram_create
 * when ctx is NULL).  The string is owned by the library. */
const char* gram_last_error(const gram_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* GRAM_H */
