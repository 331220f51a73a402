/*
 * gram_oracle.c -- CPU oracle for the GRAM encode / gradient-accumulate path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the path computes.  It shares no code, header, table or helper with the HIP
 * library and must never be called from the product path; only the tests, the
 * smoke check and the benchmark's CPU-baseline leg use it.
 *
 * Conventions (every function):
 *   - ids are int32 in [0, vocab_n); pad_id (< 0: none) marks padding.
 *   - X[vocab_n, d_in] and W[d_in, d] are float32 (dtype 0) or bfloat16 bit
 *     patterns in uint16 (dtype 1); bf16 widens exactly.  Row of X = item ID.
 *   - all sums are taken in double; callers round once to float.
 *   - return value < 0 is an error (-1 bad argument, -2 id out of range).
 *
 * Parity pins (tests/test_oracle_pins.py): brute force on tiny batches, the
 * worked example of Fig. 1 (12 interactions, 5 items), E2E == Single-step
 * (Section 4.1), the Proposition (Eq. 1-3), N = 1 reduces Multi-step to
 * Single-step (Section 4.3), library unique/matmul/scatter-add cross-checks;
 * pseudo-targets: a hand-worked case, one SGD step of rate 1 on a quadratic
 * loss lands on its target, the derivative of the pseudo-loss with respect to
 * W equals the weight gradient, pseudo-loss = half the squared norm of G;
 * content-encoder batch: with targets taken at the same weights its gradient
 * is the end-to-end gradient (Proposition), a central difference of an
 * independently written pseudo-loss matches it, a Newton step from it solves
 * a consistent regression exactly, and it vanishes at the regression's
 * solution; two-layer encoder: central differences of an independently
 * written loss, the closed form of an all-active (linear) case, gradients
 * once per unique item == once per interaction.
 * No function here is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_F32 0
#define ORC_BF16 1

static double xw_at(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORC_F32)
        return (double)((const float *)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of OpenMP threads the later calls use (n < 1: left as it is); returns the
 * number in force.  Thread count only: no arithmetic depends on it (every sum
 * below is taken by one thread in a fixed order). */
int oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
    return oracle_num_threads();
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * The set B_I of unique items of a mini-batch (Table 1; "for all i in B_I" of
 * Algorithm 1, step 1), in ascending ID order, with the index of every
 * position's item in that set and each item's multiplicity.  Padding is an
 * ordinary member of the set here; later steps give it zero rows.
 * uniq, counts: capacity >= min(m, vocab_n).  Returns U.
 */
int64_t oracle_unique(const int32_t *ids, int64_t m, int32_t vocab_n,
                      int32_t *uniq, int32_t *inverse, int32_t *counts)
{
    if (m < 0 || vocab_n <= 0) return -1;
    for (int64_t p = 0; p < m; ++p)
        if (ids[p] < 0 || ids[p] >= vocab_n) return -2;
    if (m == 0) return 0;
    int32_t *sorted = (int32_t *)malloc((size_t)m * sizeof *sorted);
    if (!sorted) return -1;
    memcpy(sorted, ids, (size_t)m * sizeof *sorted);
    qsort(sorted, (size_t)m, sizeof *sorted, cmp_i32);
    int64_t u = 0;
    for (int64_t r = 0; r < m; ++r) {
        if (r == 0 || sorted[r] != sorted[r - 1]) {
            uniq[u] = sorted[r];
            counts[u] = 0;
            ++u;
        }
        ++counts[u - 1];
    }
    free(sorted);
    for (int64_t p = 0; p < m; ++p) {
        int64_t lo = 0, hi = u - 1;           /* uniq[lo..hi] contains ids[p] */
        while (lo < hi) {
            int64_t mid = (lo + hi) / 2;
            if (uniq[mid] < ids[p]) lo = mid + 1; else hi = mid;
        }
        inverse[p] = (int32_t)lo;
    }
    return u;
}

/*
 * Same result by brute force, O(m * U): walk the positions, look every ID up
 * in the list found so far, insert new IDs at their sorted place.
 */
int64_t oracle_unique_brute(const int32_t *ids, int64_t m, int32_t vocab_n,
                            int32_t *uniq, int32_t *inverse, int32_t *counts)
{
    if (m < 0 || vocab_n <= 0) return -1;
    int64_t u = 0;
    for (int64_t p = 0; p < m; ++p) {
        int32_t v = ids[p];
        if (v < 0 || v >= vocab_n) return -2;
        int64_t j = 0;
        while (j < u && uniq[j] < v) ++j;
        if (j == u || uniq[j] != v) {
            for (int64_t t = u; t > j; --t) { uniq[t] = uniq[t - 1]; counts[t] = counts[t - 1]; }
            uniq[j] = v;
            counts[j] = 0;
            ++u;
        }
        ++counts[j];
    }
    for (int64_t p = 0; p < m; ++p) {
        int64_t j = 0;
        while (uniq[j] != ids[p]) ++j;
        inverse[p] = (int32_t)j;
    }
    return u;
}

/*
 * Content representations, once per listed item (Algorithm 1 step 1, Eq. 4),
 * with the dense linear stand-in for the encoder: E[j,:] = X[item[j],:] . W.
 * A padding item gets a zero row.  Called with item = uniq it is GRAM's
 * encode; called with item = ids (one entry per interaction) it is the
 * end-to-end forward of Section 3.3.
 */
int oracle_encode(const int32_t *item, int64_t n_items, int32_t vocab_n, int32_t pad_id,
                  const void *X, const void *W, int xw_dtype, int32_t d_in, int32_t d,
                  double *E)
{
    if (n_items < 0 || d_in <= 0 || d <= 0) return -1;
    for (int64_t j = 0; j < n_items; ++j)
        if (item[j] < 0 || item[j] >= vocab_n) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_items; ++j) {
        double *e = E + j * d;
        for (int32_t c = 0; c < d; ++c) e[c] = 0.0;
        if (item[j] == pad_id) continue;
        for (int32_t k = 0; k < d_in; ++k) {
            double x = xw_at(X, xw_dtype, (int64_t)item[j] * d_in + k);
            for (int32_t c = 0; c < d; ++c)
                e[c] += x * xw_at(W, xw_dtype, (int64_t)k * d + c);
        }
    }
    return 0;
}

/* Representation of every interaction position: H[p,:] = E[inverse[p],:]. */
int oracle_gather(const double *E, const int32_t *inverse, int64_t m, int32_t d, double *H)
{
    for (int64_t p = 0; p < m; ++p)
        memcpy(H + p * d, E + (int64_t)inverse[p] * d, (size_t)d * sizeof *H);
    return 0;
}

/*
 * Gradient of the loss with respect to each unique item's shared
 * representation (Algorithm 1 step 3, Eq. 6): the sum of dL/dH over the
 * item's occurrences, ascending position.  G is ADDED to (callers zero it for
 * a fresh batch).  The padding item's row is left untouched: whatever dH holds
 * at padded positions is ignored.
 */
int oracle_grad_accumulate(const float *dH, const int32_t *inverse, int64_t m,
                           const int32_t *uniq, int64_t u, int32_t pad_id, int32_t d,
                           double *G)
{
    for (int64_t p = 0; p < m; ++p) {
        int64_t j = inverse[p];
        if (j < 0 || j >= u) return -1;
        if (uniq[j] == pad_id) continue;
        for (int32_t c = 0; c < d; ++c)
            G[j * d + c] += (double)dH[p * d + c];
    }
    return 0;
}

/*
 * Encoder weight gradient from per-item gradients (Algorithm 1 step 4; the
 * gradient of the pseudo-loss of Eq. 7/9, which by the Proposition equals the
 * end-to-end gradient):  dW[i,c] = sum_j X[item[j], i] * G[j, c], ascending j.
 * Called with (uniq, G) it is GRAM's one-gradient-per-unique-item form; called
 * with (ids, dH widened to double) it is the per-interaction E2E form.
 * Padding items are skipped.  Threads own disjoint rows i of dW, so the
 * result does not depend on the thread count.
 */
int oracle_wgrad(const int32_t *item, int64_t n_items, int32_t vocab_n, int32_t pad_id,
                 const void *X, int xw_dtype, int32_t d_in, int32_t d,
                 const double *G, double *dW)
{
    if (n_items < 0 || d_in <= 0 || d <= 0) return -1;
    for (int64_t j = 0; j < n_items; ++j)
        if (item[j] < 0 || item[j] >= vocab_n) return -2;
    memset(dW, 0, (size_t)d_in * d * sizeof *dW);
#pragma omp parallel
    {
        int nt = 1, tid = 0;
#ifdef _OPENMP
        nt = omp_get_num_threads();
        tid = omp_get_thread_num();
#endif
        int32_t i0 = (int32_t)((int64_t)d_in * tid / nt);
        int32_t i1 = (int32_t)((int64_t)d_in * (tid + 1) / nt);
        for (int64_t j = 0; j < n_items; ++j) {
            if (item[j] == pad_id) continue;
            const double *g = G + j * d;
            for (int32_t i = i0; i < i1; ++i) {
                double x = xw_at(X, xw_dtype, (int64_t)item[j] * d_in + i);
                double *row = dW + (int64_t)i * d;
                for (int32_t c = 0; c < d; ++c) row[c] += x * g[c];
            }
        }
    }
    return 0;
}

/*
 * Selected entries of the same weight gradient, for sizes where the full
 * contraction is too slow on a CPU: out[t] = dW[rows[t], cols[t]].
 */
int oracle_wgrad_entries(const int32_t *item, int64_t n_items, int32_t vocab_n, int32_t pad_id,
                         const void *X, int xw_dtype, int32_t d_in, int32_t d,
                         const double *G, const int32_t *rows, const int32_t *cols,
                         int64_t n_entries, double *out)
{
    for (int64_t j = 0; j < n_items; ++j)
        if (item[j] < 0 || item[j] >= vocab_n) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_entries; ++t) {
        double acc = 0.0;
        for (int64_t j = 0; j < n_items; ++j) {
            if (item[j] == pad_id) continue;
            acc += xw_at(X, xw_dtype, (int64_t)item[j] * d_in + rows[t]) * G[j * d + cols[t]];
        }
        out[t] = acc;
    }
    return 0;
}

/*
 * Multi-step accumulation (Section 4.2; Algorithm 1 with N > 1): an ID-keyed
 * buffer of (count, gradient row) that persists across the N mini-batches of a
 * window.  Kept as parallel arrays sorted by ID; one batch's (uniq, counts, G)
 * is merged in.  The padding item is carried with its count and a zero row.
 * The arrays are reallocated by the merge; the caller owns the struct and
 * releases it with oracle_buffer_free.
 */
typedef struct {
    int64_t n;          /* items held */
    int32_t d;
    int32_t *ids;       /* [n] ascending */
    int64_t *counts;    /* [n] */
    double *G;          /* [n, d] */
} oracle_buffer;

oracle_buffer *oracle_buffer_new(int32_t d)
{
    oracle_buffer *b = (oracle_buffer *)calloc(1, sizeof *b);
    if (b) b->d = d;
    return b;
}

void oracle_buffer_free(oracle_buffer *b)
{
    if (!b) return;
    free(b->ids); free(b->counts); free(b->G); free(b);
}

int64_t oracle_buffer_size(const oracle_buffer *b) { return b->n; }

/* Merge (uniq ascending, counts, G rows) into the buffer; counts are 64-bit: a window of
 * epoch length (Section 4.2; the half-epoch and one-epoch periods of the experiments) can see
 * one item, the padding item above all, more than 2^31 times. */
int oracle_buffer_add64(oracle_buffer *b, const int32_t *uniq, const int64_t *counts,
                        const double *G, int64_t u)
{
    int32_t d = b->d;
    int64_t cap = b->n + u;
    int32_t *ids = (int32_t *)malloc((size_t)(cap ? cap : 1) * sizeof *ids);
    int64_t *cnt = (int64_t *)malloc((size_t)(cap ? cap : 1) * sizeof *cnt);
    double *g = (double *)malloc((size_t)(cap ? cap : 1) * d * sizeof *g);
    if (!ids || !cnt || !g) { free(ids); free(cnt); free(g); return -1; }
    int64_t a = 0, c = 0, n = 0;
    while (a < b->n || c < u) {
        int take_old = a < b->n && (c >= u || b->ids[a] <= uniq[c]);
        int take_new = c < u && (a >= b->n || uniq[c] <= b->ids[a]);
        ids[n] = take_old ? b->ids[a] : uniq[c];
        cnt[n] = 0;
        for (int32_t k = 0; k < d; ++k) g[n * d + k] = 0.0;
        if (take_old) {
            cnt[n] += b->counts[a];
            for (int32_t k = 0; k < d; ++k) g[n * d + k] += b->G[a * d + k];
        }
        if (take_new) {
            cnt[n] += counts[c];
            for (int32_t k = 0; k < d; ++k) g[n * d + k] += G[c * d + k];
        }
        a += take_old; c += take_new; ++n;
    }
    free(b->ids); free(b->counts); free(b->G);
    b->ids = ids; b->counts = cnt; b->G = g; b->n = n;
    return 0;
}

int oracle_buffer_add(oracle_buffer *b, const int32_t *uniq, const int32_t *counts,
                      const double *G, int64_t u)
{
    int64_t *wide = (int64_t *)malloc((size_t)(u ? u : 1) * sizeof *wide);
    if (!wide) return -1;
    for (int64_t j = 0; j < u; ++j) wide[j] = counts[j];
    int rc = oracle_buffer_add64(b, uniq, wide, G, u);
    free(wide);
    return rc;
}

/* Copy the buffer out (ascending ID).  Any pointer may be NULL. */
int oracle_buffer_export(const oracle_buffer *b, int32_t *ids, int64_t *counts, double *G)
{
    if (ids) memcpy(ids, b->ids, (size_t)b->n * sizeof *ids);
    if (counts) memcpy(counts, b->counts, (size_t)b->n * sizeof *counts);
    if (G) memcpy(G, b->G, (size_t)b->n * b->d * sizeof *G);
    return 0;
}

/* Rows of the buffer for the given IDs (ascending or not): G_out[j,:] = the
 * gradient accumulated so far for ids[j], zeros for an ID the buffer does not
 * hold. */
int oracle_buffer_rows(const oracle_buffer *b, const int32_t *ids, int64_t u, double *G_out)
{
    for (int64_t j = 0; j < u; ++j) {
        int64_t lo = 0, hi = b->n;                 /* first entry >= ids[j] */
        while (lo < hi) {
            int64_t mid = lo + (hi - lo) / 2;
            if (b->ids[mid] < ids[j]) lo = mid + 1; else hi = mid;
        }
        int found = lo < b->n && b->ids[lo] == ids[j];
        for (int32_t k = 0; k < b->d; ++k) G_out[j * b->d + k] = found ? b->G[lo * b->d + k] : 0.0;
    }
    return 0;
}

/*
 * Pseudo-targets (Algorithm 1 step 3, Eq. 6): the representation of an item is
 * treated as a trainable embedding and moved by one plain gradient step of
 * rate 1, h~_i = h_i - grad L(h_i), where grad L(h_i) is the gradient
 * accumulated for item i (all its occurrences; all steps of the window so far,
 * Section 4.2).  The pseudo-loss of Eq. 7 at the current encoder is
 * 1/2 sum_i |h~_i - h_i|^2.  E, G, Ht are [u, d]; *loss receives the scalar.
 */
int oracle_pseudo_target(const double *E, const double *G, int64_t u, int32_t d, double *Ht,
                         double *loss)
{
    double total = 0.0;
    for (int64_t j = 0; j < u; ++j)
        for (int32_t k = 0; k < d; ++k) {
            double target = E[j * d + k] - G[j * d + k];
            double miss = target - E[j * d + k];
            Ht[j * d + k] = target;
            total += 0.5 * miss * miss;
        }
    *loss = total;
    return 0;
}

/*
 * One content-encoder batch of the update of Algorithm 1 step 4: the encoder
 * is regressed towards the stored pseudo-targets of the listed items (Eq. 7;
 * the content-encoder batch size of the GPU-memory table says that this update
 * runs over the accumulated items a chunk at a time).  With the encoder's
 * CURRENT weights W, which may have moved since the targets were taken,
 *   h_j    = X[item[j],:] . W                         (Eq. 4)
 *   miss_j = h_j - Ht[j,:]
 *   loss   = 1/2 sum_j |Ht[j,:] - h_j|^2              (Eq. 7)
 *   dW     = d loss / d W = sum_j X[item[j],:]^T miss_j
 * A padding item takes no part: zero miss row, nothing added to loss or dW.
 * miss is [n, d], dW is [d_in, d]; *loss receives the scalar.
 */
int oracle_pseudo_loss_grad(const int32_t *item, int64_t n_items, int32_t vocab_n, int32_t pad_id,
                            const void *X, const void *W, int xw_dtype, int32_t d_in, int32_t d,
                            const double *Ht, double *miss, double *loss, double *dW)
{
    int rc = oracle_encode(item, n_items, vocab_n, pad_id, X, W, xw_dtype, d_in, d, miss);
    if (rc < 0) return rc;
    double total = 0.0;
    for (int64_t j = 0; j < n_items; ++j)
        for (int32_t c = 0; c < d; ++c) {
            double r = item[j] == pad_id ? 0.0 : miss[j * d + c] - Ht[j * d + c];
            miss[j * d + c] = r;
            total += 0.5 * r * r;
        }
    *loss = total;
    return oracle_wgrad(item, n_items, vocab_n, pad_id, X, xw_dtype, d_in, d, miss, dW);
}

/*
 * A deeper stand-in for the content encoder: two dense layers with a rectifier,
 *   z_j = X[item[j],:] . W1      a_j = max(z_j, 0)      h_j = a_j . W2,
 * W1 [d_in, d_hid], W2 [d_hid, d].  Nothing in the method depends on the encoder
 * being linear (Eq. 4 takes any CE; the Proposition holds for any f); the hidden
 * activation a_j is what a training framework keeps for the backward pass, once
 * per listed item: per unique item under GRAM, per interaction end to end (the
 * memory argument of the section on GPU memory consumption).
 * A padding item gets zero rows.  A1 (nullable) [n, d_hid], E [n, d].
 */
int oracle_mlp_encode(const int32_t *item, int64_t n_items, int32_t vocab_n, int32_t pad_id,
                      const void *X, const void *W1, const void *W2, int xw_dtype, int32_t d_in,
                      int32_t d_hid, int32_t d, double *A1, double *E)
{
    if (n_items < 0 || d_in <= 0 || d_hid <= 0 || d <= 0) return -1;
    for (int64_t j = 0; j < n_items; ++j)
        if (item[j] < 0 || item[j] >= vocab_n) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_items; ++j) {
        double *a = (double *)calloc((size_t)d_hid, sizeof *a);
        double *e = E + j * d;
        for (int32_t c = 0; c < d; ++c) e[c] = 0.0;
        if (item[j] != pad_id) {
            for (int32_t k = 0; k < d_in; ++k) {
                double x = xw_at(X, xw_dtype, (int64_t)item[j] * d_in + k);
                for (int32_t q = 0; q < d_hid; ++q) a[q] += x * xw_at(W1, xw_dtype, (int64_t)k * d_hid + q);
            }
            for (int32_t q = 0; q < d_hid; ++q) {
                if (a[q] < 0.0) a[q] = 0.0;
                for (int32_t c = 0; c < d; ++c) e[c] += a[q] * xw_at(W2, xw_dtype, (int64_t)q * d + c);
            }
        }
        if (A1) memcpy(A1 + j * d_hid, a, (size_t)d_hid * sizeof *a);
        free(a);
    }
    return 0;
}

/*
 * Backward pass of the same encoder for the listed items, given the gradient
 * with respect to each item's output, R [n, d] (the accumulated gradient G of
 * Eq. 6, or the regression miss of Eq. 7):
 *   dW2 = sum_j a_j^T R_j       da_j = R_j . W2^T       dz_j = da_j where z_j > 0, else 0
 *   dW1 = sum_j X[item[j],:]^T dz_j
 * Items are visited in ascending j; a padding item is skipped.
 */
int oracle_mlp_grad(const int32_t *item, int64_t n_items, int32_t vocab_n, int32_t pad_id,
                    const void *X, const void *W1, const void *W2, int xw_dtype, int32_t d_in,
                    int32_t d_hid, int32_t d, const double *R, double *dW1, double *dW2)
{
    if (n_items < 0 || d_in <= 0 || d_hid <= 0 || d <= 0) return -1;
    for (int64_t j = 0; j < n_items; ++j)
        if (item[j] < 0 || item[j] >= vocab_n) return -2;
    memset(dW1, 0, (size_t)d_in * d_hid * sizeof *dW1);
    memset(dW2, 0, (size_t)d_hid * d * sizeof *dW2);
    double *z = (double *)malloc((size_t)d_hid * sizeof *z);
    double *dz = (double *)malloc((size_t)d_hid * sizeof *dz);
    if (!z || !dz) { free(z); free(dz); return -1; }
    for (int64_t j = 0; j < n_items; ++j) {
        if (item[j] == pad_id) continue;
        const double *r = R + j * d;
        for (int32_t q = 0; q < d_hid; ++q) z[q] = 0.0;
        for (int32_t k = 0; k < d_in; ++k) {
            double x = xw_at(X, xw_dtype, (int64_t)item[j] * d_in + k);
            for (int32_t q = 0; q < d_hid; ++q) z[q] += x * xw_at(W1, xw_dtype, (int64_t)k * d_hid + q);
        }
        for (int32_t q = 0; q < d_hid; ++q) {
            double a = z[q] > 0.0 ? z[q] : 0.0;
            double da = 0.0;
            for (int32_t c = 0; c < d; ++c) {
                dW2[(int64_t)q * d + c] += a * r[c];
                da += r[c] * xw_at(W2, xw_dtype, (int64_t)q * d + c);
            }
            dz[q] = z[q] > 0.0 ? da : 0.0;
        }
        for (int32_t k = 0; k < d_in; ++k) {
            double x = xw_at(X, xw_dtype, (int64_t)item[j] * d_in + k);
            for (int32_t q = 0; q < d_hid; ++q) dW1[(int64_t)k * d_hid + q] += x * dz[q];
        }
    }
    free(z); free(dz);
    return 0;
}

/*
 * Selected entries of the two-layer encoder's weight gradients, for sizes where
 * the full backward pass is too slow on a CPU:
 *   out1[t] = dW1[i1[t], q1[t]] = sum_j X[item[j], i1] * [z_j[q1] > 0] * (R_j . W2[q1,:])
 *   out2[t] = dW2[q2[t], c2[t]] = sum_j max(z_j[q2], 0) * R[j, c2]
 * with z_j[q] = X[item[j],:] . W1[:,q]; padding items are skipped.
 */
int oracle_mlp_grad_entries(const int32_t *item, int64_t n_items, int32_t vocab_n, int32_t pad_id,
                            const void *X, const void *W1, const void *W2, int xw_dtype, int32_t d_in,
                            int32_t d_hid, int32_t d, const double *R, const int32_t *i1,
                            const int32_t *q1, int64_t n1, double *out1, const int32_t *q2,
                            const int32_t *c2, int64_t n2, double *out2)
{
    for (int64_t j = 0; j < n_items; ++j)
        if (item[j] < 0 || item[j] >= vocab_n) return -2;
#pragma omp parallel for schedule(dynamic)
    for (int64_t t = 0; t < n1 + n2; ++t) {
        const int first = t < n1;
        const int32_t q = first ? q1[t] : q2[t - n1];
        double acc = 0.0;
        for (int64_t j = 0; j < n_items; ++j) {
            if (item[j] == pad_id) continue;
            double z = 0.0;
            for (int32_t k = 0; k < d_in; ++k)
                z += xw_at(X, xw_dtype, (int64_t)item[j] * d_in + k) * xw_at(W1, xw_dtype, (int64_t)k * d_hid + q);
            if (first) {
                if (z > 0.0) {
                    double da = 0.0;
                    for (int32_t c = 0; c < d; ++c) da += R[j * d + c] * xw_at(W2, xw_dtype, (int64_t)q * d + c);
                    acc += xw_at(X, xw_dtype, (int64_t)item[j] * d_in + i1[t]) * da;
                }
            } else if (z > 0.0) {
                acc += z * R[j * d + c2[t - n1]];
            }
        }
        if (first) out1[t] = acc; else out2[t - n1] = acc;
    }
    return 0;
}
