/*
 * CPU oracle for the hot-embedding path of the FAE method (arxiv 2103.00686).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, by-eye-checkable
 * definition of what the path computes.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the product (the HIP library) shares
 * no code with it and never routes through it.
 *
 * Every function is a naive loop over host arrays.  Floating-point sums are
 * accumulated in double in the order the definition states and rounded to fp32
 * once.  Nothing here is blocked, fused, vectorised or reordered.
 *
 * Pins (tests/test_oracle_pins.py): brute-force counts, the worked example of
 * Eq. 1 (Sec. 4.1.2), hot+cold = all rows, set-membership partition, the
 * closed form p^B of Sec. 3 (1), dense matrix forms of pooling and of the
 * gradient, bit-exact integer-valued cases, PyTorch-CPU's stock embedding-bag
 * as a black-box cross-check.  No function in this file is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ERANGE (-2)
#define ORC_ENOSPC (-3)

/* ------------------------------------------------------------------ */
/* Embedding Logger (Sec. 4.1.2): k = number of accesses of the        */
/* sampled inputs to every row of one table.                           */
/* ------------------------------------------------------------------ */
int orc_histogram(int64_t n_rows, const int32_t *idx, int64_t n, uint32_t *cnt)
{
    for (int64_t j = 0; j < n; ++j) {
        if (idx[j] < 0 || (int64_t)idx[j] >= n_rows)
            return ORC_ERANGE;
    }
    for (int64_t j = 0; j < n; ++j)
        cnt[idx[j]] += 1u;
    return ORC_OK;
}

/* Eq. 1: H_zt = t * T * x/100, with t given in per cent (the worked example of
 * Sec. 4.1.2 only holds with t = 1e-2 read as a percentage). */
double orc_cutoff_eq1(double t_percent, double T, double x_percent)
{
    return (t_percent / 100.0) * T * (x_percent / 100.0);
}

/* Smallest integer count that satisfies k >= H (Eq. 2 uses >=).  A relative
 * guard of 1e-12 keeps an H that is an integer up to rounding from moving up. */
uint32_t orc_cutoff_int(double H)
{
    if (H <= 0.0)
        return 0u;
    double c = ceil(H * (1.0 - 1e-12));
    if (c > 4294967295.0)
        return 4294967295u;
    return (uint32_t)c;
}

/* Number of rows with k >= H (Eq. 2 summed over the whole logger). */
int64_t orc_count_hot(const uint32_t *cnt, int64_t n_rows, uint32_t H)
{
    int64_t n = 0;
    for (int64_t r = 0; r < n_rows; ++r)
        if (cnt[r] >= H)
            n += 1;
    return n;
}

/* ------------------------------------------------------------------ */
/* Estimating the hot size from sampled chunks of the logger           */
/* (Sec. 4.1.2, "Estimating the hot embedding table sizes per          */
/* threshold" and "Confidence in the estimated embedding table size"). */
/* The chunk numbers are inputs: the caller draws them, without        */
/* replacement, from the N = ceil(n_rows / m) aligned chunks of m      */
/* consecutive logger entries.                                         */
/* ------------------------------------------------------------------ */

/* Eq. 2: C_i = number of entries of chunk i with k >= H.  The last chunk of a
 * table may hold fewer than m entries; the missing ones count as not hot. */
int64_t orc_chunk_count(const uint32_t *cnt, int64_t n_rows, int64_t m,
                        int64_t chunk, uint32_t H)
{
    int64_t C = 0;
    for (int64_t j = 0; j < m; ++j) {
        int64_t r = chunk * m + j;
        if (r < n_rows && cnt[r] >= H)
            C += 1;
    }
    return C;
}

/* Eq. 3: mean of the n chunk counts, and their standard deviation s (the
 * sample standard deviation, divisor n - 1, as the t-interval takes it). */
void orc_mean_std(const int64_t *Ci, int64_t n, double *ybar, double *s)
{
    double sum = 0.0;
    for (int64_t i = 0; i < n; ++i)
        sum += (double)Ci[i];
    *ybar = sum / (double)n;
    double ss = 0.0;
    for (int64_t i = 0; i < n; ++i)
        ss += ((double)Ci[i] - *ybar) * ((double)Ci[i] - *ybar);
    *s = n > 1 ? sqrt(ss / (double)(n - 1)) : 0.0;
}

/* Eq. 4: half-width of the confidence interval of the mean,
 * t_{alpha/2} * sqrt(((N - n) / N) * (s^2 / n)); the caller supplies the
 * quantile t_{alpha/2} of Student's t with n - 1 degrees of freedom. */
double orc_ci_halfwidth(double s, int64_t n, int64_t N, double t_quantile)
{
    return t_quantile * sqrt(((double)(N - n) / (double)N) * (s * s / (double)n));
}

/* ceil(c * T / n) in exact integer arithmetic (c*T < 2^63 is a precondition). */
static uint32_t scaled_cutoff(int64_t c, int64_t T, int64_t n)
{
    int64_t v = (c * T + n - 1) / n;
    if (v > 4294967295LL)
        v = 4294967295LL;
    return (uint32_t)v;
}

/* Budget mode (Sec. 4.1: "the top h entries that fit L", expressed through one
 * count threshold as the paper's t is).  Tables smaller than small_table_bytes
 * are wholly hot (Sec. 4.1.2, Embedding Logger); every other table z uses the
 * cutoff H_z(c) = ceil(c * T_z / t_denom), i.e. the threshold t = c / t_denom as a
 * fraction of the table's accesses T_z (Sec. 4.1: hot entries have >= t * T accesses);
 * the answer is the smallest c >= 0 whose hot rows (small tables included) fit
 * budget_bytes.  The caller fixes the grid of t through t_denom. */
int orc_budget_cutoff(int32_t n_tables, int32_t dim, const int64_t *rows,
                      const uint32_t *const *cnt, const int64_t *T,
                      int64_t t_denom, int64_t budget_bytes,
                      int64_t small_table_bytes, int64_t *c_out,
                      uint32_t *H_out, int64_t *n_hot_out)
{
    if (n_tables <= 0 || dim <= 0 || t_denom <= 0)
        return ORC_EINVAL;
    int64_t row_bytes = (int64_t)dim * 4;
    uint32_t max_cnt = 0;
    for (int32_t z = 0; z < n_tables; ++z)
        for (int64_t r = 0; r < rows[z]; ++r)
            if (cnt[z][r] > max_cnt)
                max_cnt = cnt[z][r];
    for (int64_t c = 0;; ++c) {
        int64_t bytes = 0;
        int all_above = 1;
        for (int32_t z = 0; z < n_tables; ++z) {
            uint32_t H;
            if (rows[z] * row_bytes < small_table_bytes)
                H = 0u;
            else
                H = scaled_cutoff(c, T[z], t_denom);
            if (H != 0u && H <= max_cnt)
                all_above = 0;
            H_out[z] = H;
            n_hot_out[z] = orc_count_hot(cnt[z], rows[z], H);
            bytes += n_hot_out[z] * row_bytes;
        }
        if (bytes <= budget_bytes) {
            *c_out = c;
            return ORC_OK;
        }
        if (c > 0 && all_above)
            return ORC_ENOSPC; /* only the small tables are left and they do not fit */
    }
}

/* Embedding Classifier (Sec. 4.2): one pass over the logger, tag each row hot
 * or cold; hot rows get consecutive slots in ascending row order. */
int64_t orc_classify(const uint32_t *cnt, int64_t n_rows, uint32_t H,
                     int32_t *remap, int32_t *hot_ids)
{
    int64_t slot = 0;
    for (int64_t r = 0; r < n_rows; ++r) {
        if (cnt[r] >= H) {
            remap[r] = (int32_t)slot;
            hot_ids[slot] = (int32_t)r;
            slot += 1;
        } else {
            remap[r] = -1;
        }
    }
    return slot;
}

/* Embedding Replicator (Sec. 4): extract the hot rows into their own table. */
void orc_gather_rows(const float *W, int32_t dim, const int32_t *hot_ids,
                     int64_t n_hot, float *hotW)
{
    for (int64_t s = 0; s < n_hot; ++s)
        for (int32_t c = 0; c < dim; ++c)
            hotW[s * dim + c] = W[(int64_t)hot_ids[s] * dim + c];
}

/* Embedding synchronisation when training switches from hot to cold mini-batches
 * (Sec. 3 (4); Sec. 6.2, "Embedding Synchronization"): the updated hot rows go back to
 * their places in the full table; every other row of the full table stays as it is.
 * The opposite direction is orc_gather_rows. */
void orc_scatter_rows(float *W, int32_t dim, const int32_t *hot_ids,
                      int64_t n_hot, const float *hotW)
{
    for (int64_t s = 0; s < n_hot; ++s)
        for (int32_t c = 0; c < dim; ++c)
            W[(int64_t)hot_ids[s] * dim + c] = hotW[s * dim + c];
}

/* Procedural initial weights of a virtual table (counter-based; the synthetic
 * workloads define it): u24 = top 24 bits of a 64-bit mix of (seed, table,
 * row*dim+col+1); w = (u24 * 2^-24 - 0.5) * 0.1 in fp32. */
static uint64_t orc_mix64(uint64_t x)
{
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ULL;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBULL;
    x ^= x >> 31;
    return x;
}

float orc_w0(uint64_t seed, int32_t table, int64_t row, int32_t dim, int32_t col)
{
    uint64_t key = orc_mix64(seed ^ (0x9E3779B97F4A7C15ULL * (uint64_t)(table + 1)));
    uint64_t ctr = (uint64_t)row * (uint64_t)dim + (uint64_t)col + 1u;
    uint64_t h = orc_mix64(key + 0xD1B54A32D192ED03ULL * ctr);
    volatile float u = (float)(uint32_t)(h >> 40);
    volatile float v = u * 0x1p-24f - 0.5f;
    volatile float w = v * 0.1f;
    return w;
}

void orc_w0_rows(uint64_t seed, int32_t table, const int64_t *rows, int64_t n,
                 int32_t dim, float *out)
{
    for (int64_t i = 0; i < n; ++i)
        for (int32_t c = 0; c < dim; ++c)
            out[i * dim + c] = orc_w0(seed, table, rows[i], dim, c);
}

/* Input Classifier (Sec. 4.2): a sparse input is hot iff every access in every
 * table goes to a hot row.  Samples keep their order inside the hot and the cold
 * list; for hot samples the hot slots and the rebuilt CSR offsets are emitted.
 * offsets[z] == NULL means one lookup per sample in table z. */
int orc_partition(int32_t n_tables, const int64_t *rows, int64_t n_samples,
                  const int32_t *const *idx, const int32_t *const *offsets,
                  const int32_t *const *remap, int32_t *hot_samples,
                  int32_t *cold_samples, int64_t *n_hot_samples,
                  int32_t *const *slots_out, int32_t *const *hoffsets_out)
{
    int64_t nh = 0, nc = 0;
    for (int32_t z = 0; z < n_tables; ++z)
        hoffsets_out[z][0] = 0;
    for (int64_t s = 0; s < n_samples; ++s) {
        int hot = 1;
        for (int32_t z = 0; z < n_tables; ++z) {
            int64_t b = offsets[z] ? offsets[z][s] : s;
            int64_t e = offsets[z] ? offsets[z][s + 1] : s + 1;
            if (e < b)
                return ORC_ERANGE;
            for (int64_t j = b; j < e; ++j) {
                int32_t r = idx[z][j];
                if (r < 0 || (int64_t)r >= rows[z])
                    return ORC_ERANGE;
                if (remap[z][r] < 0)
                    hot = 0;
            }
        }
        if (!hot) {
            cold_samples[nc++] = (int32_t)s;
            continue;
        }
        for (int32_t z = 0; z < n_tables; ++z) {
            int64_t b = offsets[z] ? offsets[z][s] : s;
            int64_t e = offsets[z] ? offsets[z][s + 1] : s + 1;
            int64_t w = hoffsets_out[z][nh];
            for (int64_t j = b; j < e; ++j)
                slots_out[z][w++] = remap[z][idx[z][j]];
            hoffsets_out[z][nh + 1] = (int32_t)w;
        }
        hot_samples[nh++] = (int32_t)s;
    }
    *n_hot_samples = nh;
    return ORC_OK;
}

/* Hot mini-batch forward for one table: sum pooling of the rows a bag names,
 * with multiplicity; an empty bag gives zeros.  out/mag rows are `stride`
 * elements apart; mag (optional) receives sum |term| for the tolerance. */
int orc_embbag_fwd(int64_t n_hot, int32_t dim, const float *hotW,
                   int64_t n_samples, const int32_t *slots,
                   const int32_t *offsets, float *out, int64_t out_stride,
                   double *mag, int64_t mag_stride)
{
    for (int64_t s = 0; s < n_samples; ++s) {
        int64_t b = offsets ? offsets[s] : s;
        int64_t e = offsets ? offsets[s + 1] : s + 1;
        for (int32_t c = 0; c < dim; ++c) {
            double acc = 0.0, m = 0.0;
            for (int64_t j = b; j < e; ++j) {
                if (slots[j] < 0 || (int64_t)slots[j] >= n_hot)
                    return ORC_ERANGE;
                double v = (double)hotW[(int64_t)slots[j] * dim + c];
                acc += v;
                m += fabs(v);
            }
            out[s * out_stride + c] = (float)acc;
            if (mag)
                mag[s * mag_stride + c] = m;
        }
    }
    return ORC_OK;
}

/* bag_of[j] = sample whose bag holds lookup j. */
void orc_bag_of(const int32_t *offsets, int64_t n_samples, int32_t *bag_of)
{
    for (int64_t s = 0; s < n_samples; ++s) {
        int64_t b = offsets ? offsets[s] : s;
        int64_t e = offsets ? offsets[s + 1] : s + 1;
        for (int64_t j = b; j < e; ++j)
            bag_of[j] = (int32_t)s;
    }
}

/* Stable sort of the lookup positions 0..n-1 by slot (bottom-up merge sort:
 * on equal slots the left run wins, so equal slots keep position order). */
int orc_sort_by_slot(const int32_t *slots, int64_t n, int32_t *order)
{
    int32_t *tmp = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    if (!tmp)
        return ORC_ENOSPC;
    for (int64_t i = 0; i < n; ++i)
        order[i] = (int32_t)i;
    for (int64_t w = 1; w < n; w *= 2) {
        for (int64_t lo = 0; lo < n; lo += 2 * w) {
            int64_t mid = lo + w < n ? lo + w : n;
            int64_t hi = lo + 2 * w < n ? lo + 2 * w : n;
            int64_t a = lo, b = mid, k = lo;
            while (a < mid && b < hi) {
                if (slots[order[b]] < slots[order[a]])
                    tmp[k++] = order[b++];
                else
                    tmp[k++] = order[a++];
            }
            while (a < mid)
                tmp[k++] = order[a++];
            while (b < hi)
                tmp[k++] = order[b++];
        }
        memcpy(order, tmp, (size_t)n * sizeof(int32_t));
    }
    free(tmp);
    return ORC_OK;
}

/* Distinct slots in ascending order and how often each occurs. */
int64_t orc_runs(const int32_t *slots, const int32_t *order, int64_t n,
                 int32_t *uniq, int32_t *runlen)
{
    int64_t u = 0;
    for (int64_t i = 0; i < n; ++i) {
        int32_t s = slots[order[i]];
        if (u > 0 && uniq[u - 1] == s) {
            runlen[u - 1] += 1;
        } else {
            uniq[u] = s;
            runlen[u] = 1;
            u += 1;
        }
    }
    return u;
}

/* Summed gradient of selected runs: G[i] = sum over the lookups of run sel[i],
 * in sorted order, of the upstream gradient row of the lookup's bag.  gout
 * points at this table's first column; rows are gout_stride floats apart.
 * run_start[u] is the first sorted position of run u. */
void orc_run_grads(const int32_t *order, const int32_t *bag_of,
                   const int64_t *run_start, const int32_t *runlen,
                   const int64_t *sel, int64_t n_sel, const float *gout,
                   int64_t gout_stride, int32_t dim, double *G, double *Gabs)
{
    for (int64_t i = 0; i < n_sel; ++i) {
        int64_t u = sel[i];
        for (int32_t c = 0; c < dim; ++c) {
            double acc = 0.0, m = 0.0;
            for (int64_t p = run_start[u]; p < run_start[u] + runlen[u]; ++p) {
                double g = (double)gout[(int64_t)bag_of[order[p]] * gout_stride + c];
                acc += g;
                m += fabs(g);
            }
            G[i * dim + c] = acc;
            if (Gabs)
                Gabs[i * dim + c] = m;
        }
    }
}

/* Plain SGD on n rows: w <- w - lr * G, computed in double, rounded once. */
void orc_sgd_rows(float *W_rows, const double *G, float lr, int64_t n, int32_t dim)
{
    for (int64_t i = 0; i < n * dim; ++i)
        W_rows[i] = (float)((double)W_rows[i] - (double)lr * G[i]);
}

/* Hot mini-batch backward + optimizer for one table on a materialised hot
 * table: sort lookups by slot, sum the gradients of duplicates, one SGD update
 * per distinct row with the summed gradient; all other rows stay untouched.
 * uniq/runlen need room for n_lookups entries.  mag (optional, [U][dim]) gets
 * |w_old| + lr * sum |g| for the tolerance. */
int orc_embbag_bwd_sgd(int64_t n_hot, int32_t dim, float *hotW,
                       int64_t n_samples, const int32_t *slots,
                       const int32_t *offsets, int64_t n_lookups,
                       const float *gout, int64_t gout_stride, float lr,
                       int32_t *uniq, int32_t *runlen, int64_t *n_uniq,
                       double *mag)
{
    int64_t n = n_lookups;
    for (int64_t j = 0; j < n; ++j)
        if (slots[j] < 0 || (int64_t)slots[j] >= n_hot)
            return ORC_ERANGE;
    int32_t *order = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    int32_t *bag = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    double *G = (double *)malloc((size_t)dim * sizeof(double));
    double *Ga = (double *)malloc((size_t)dim * sizeof(double));
    if (!order || !bag || !G || !Ga)
        return ORC_ENOSPC;
    orc_bag_of(offsets, n_samples, bag);
    int rc = orc_sort_by_slot(slots, n, order);
    if (rc != ORC_OK)
        return rc;
    int64_t U = orc_runs(slots, order, n, uniq, runlen);
    int64_t start = 0;
    for (int64_t u = 0; u < U; ++u) {
        int64_t sel = 0;
        int64_t rs = start;
        /* one run at a time: run_start/runlen arrays of length 1 */
        int32_t rl = runlen[u];
        orc_run_grads(order, bag, &rs, &rl, &sel, 1, gout, gout_stride, dim, G, Ga);
        float *row = hotW + (int64_t)uniq[u] * dim;
        if (mag)
            for (int32_t c = 0; c < dim; ++c)
                mag[u * dim + c] = fabs((double)row[c]) + (double)lr * Ga[c];
        orc_sgd_rows(row, G, lr, 1, dim);
        start += runlen[u];
    }
    *n_uniq = U;
    free(order);
    free(bag);
    free(G);
    free(Ga);
    return ORC_OK;
}


/* ------------------------------------------------------------------ */
/* Variants the paper leaves open (Sec. 2.2 names the pooled lookup    */
/* and the optimizer step without fixing either): mean pooling and a   */
/* row-wise Adagrad optimizer.                                         */
/* ------------------------------------------------------------------ */

/* Mean pooling: the sum of the bag's rows (with multiplicity) divided by the
 * number of lookups in the bag; an empty bag gives zeros.  mag (optional)
 * receives sum |term| / len for the tolerance. */
int orc_embbag_fwd_mean(int64_t n_hot, int32_t dim, const float *hotW,
                        int64_t n_samples, const int32_t *slots,
                        const int32_t *offsets, float *out, int64_t out_stride,
                        double *mag, int64_t mag_stride)
{
    for (int64_t s = 0; s < n_samples; ++s) {
        int64_t b = offsets ? offsets[s] : s;
        int64_t e = offsets ? offsets[s + 1] : s + 1;
        for (int32_t c = 0; c < dim; ++c) {
            double acc = 0.0, m = 0.0;
            for (int64_t j = b; j < e; ++j) {
                if (slots[j] < 0 || (int64_t)slots[j] >= n_hot)
                    return ORC_ERANGE;
                double v = (double)hotW[(int64_t)slots[j] * dim + c];
                acc += v;
                m += fabs(v);
            }
            if (e > b) {
                acc /= (double)(e - b);
                m /= (double)(e - b);
            }
            out[s * out_stride + c] = (float)acc;
            if (mag)
                mag[s * mag_stride + c] = m;
        }
    }
    return ORC_OK;
}

/* Gradient of a row under mean pooling: every lookup of a bag of len lookups
 * receives the bag's upstream gradient divided by len.  Same arguments as
 * orc_run_grads plus bag_len[s]. */
void orc_run_grads_mean(const int32_t *order, const int32_t *bag_of,
                        const int32_t *bag_len, const int64_t *run_start,
                        const int32_t *runlen, const int64_t *sel,
                        int64_t n_sel, const float *gout, int64_t gout_stride,
                        int32_t dim, double *G, double *Gabs)
{
    for (int64_t i = 0; i < n_sel; ++i) {
        int64_t u = sel[i];
        for (int32_t c = 0; c < dim; ++c) {
            double acc = 0.0, m = 0.0;
            for (int64_t p = run_start[u]; p < run_start[u] + runlen[u]; ++p) {
                int32_t s = bag_of[order[p]];
                double g = (double)gout[(int64_t)s * gout_stride + c] / (double)bag_len[s];
                acc += g;
                m += fabs(g);
            }
            G[i * dim + c] = acc;
            if (Gabs)
                Gabs[i * dim + c] = m;
        }
    }
}

/* Row-wise Adagrad on n rows, one accumulator per row: the accumulator grows by
 * the mean over the row's elements of the squared gradient, and the row moves
 * by lr * G / (sqrt(accumulator) + eps).  Computed in double, rounded once. */
void orc_rowwise_adagrad_rows(float *W_rows, float *state, const double *G,
                              float lr, float eps, int64_t n, int32_t dim)
{
    for (int64_t i = 0; i < n; ++i) {
        double ms = 0.0;
        for (int32_t c = 0; c < dim; ++c)
            ms += G[i * dim + c] * G[i * dim + c];
        ms /= (double)dim;
        double acc = (double)state[i] + ms;
        double scale = (double)lr / (sqrt(acc) + (double)eps);
        state[i] = (float)acc;
        for (int32_t c = 0; c < dim; ++c)
            W_rows[i * dim + c] = (float)((double)W_rows[i * dim + c] - scale * G[i * dim + c]);
    }
}
