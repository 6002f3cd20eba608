// Hot-size estimate from sampled chunks of the logger, its confidence interval, and the
// threshold search on the sampled logger (Sec. 4.1.2: "Estimating the hot embedding table
// sizes per threshold", Eq. 2-4, and "Converging on a Threshold using Statistical
// Optimizer").
//
// Device work: one workgroup per sampled chunk counts the entries with k >= H (Eq. 2).
// With n = 35 chunks of m = 1024 entries per table that is 140 KiB of reads per table and
// threshold, so a probe of the search costs a launch and a read-back, not a table scan.
// Host work (fp64, at most FAE_MAX_TABLES * n numbers): mean, standard deviation, the
// Student-t quantile and the interval (Eq. 3, Eq. 4).
#include "fae_internal.h"

#include <math.h>

#include <algorithm>

#define EST_THREADS 256

struct EstArgs {
    const uint32_t *counts[FAE_MAX_TABLES];
    int64_t rows[FAE_MAX_TABLES];
    uint32_t cutoff[FAE_MAX_TABLES];
    int32_t chunk_start[FAE_MAX_TABLES + 1]; // prefix of sampled chunks per table
    const int64_t *chunks;                   // device, all tables' chunk numbers, table after table
    int32_t *C;                              // device, one count per sampled chunk
    int64_t m;
    int32_t n_tables;
};

__global__ __launch_bounds__(EST_THREADS) void est_chunk_count_kernel(EstArgs a)
{
    __shared__ int s_part[EST_THREADS / FAE_WAVE];
    const int z = fae_find_table(a.chunk_start, a.n_tables, blockIdx.x);
    const int64_t first = a.chunks[blockIdx.x] * a.m;
    int64_t last = first + a.m;
    if (last > a.rows[z])
        last = a.rows[z]; // a short last chunk: the missing entries are not hot
    const uint32_t H = a.cutoff[z];
    const uint32_t *k = a.counts[z];
    int c = 0;
    for (int64_t r = first + threadIdx.x; r < last; r += EST_THREADS)
        c += k[r] >= H ? 1 : 0;
#pragma unroll
    for (int d = FAE_WAVE / 2; d > 0; d >>= 1)
        c += __shfl_xor(c, d, FAE_WAVE);
    if (fae_lane() == 0)
        s_part[threadIdx.x / FAE_WAVE] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int w = 0; w < EST_THREADS / FAE_WAVE; ++w)
            t += s_part[w];
        a.C[blockIdx.x] = t;
    }
}

// ---------------------------------------------------------------------------------
// Student's t quantile (host): the CDF through the regularised incomplete beta function
// (continued fraction, modified Lentz), inverted by bisection.
// ---------------------------------------------------------------------------------
namespace {
double beta_cf(double a, double b, double x)
{
    const double tiny = 1e-300;
    double c = 1.0, d = 1.0 - (a + b) * x / (a + 1.0);
    if (fabs(d) < tiny)
        d = tiny;
    d = 1.0 / d;
    double h = d;
    for (int i = 1; i <= 500; ++i) {
        const double i2 = 2.0 * i;
        double num = i * (b - i) * x / ((a + i2 - 1.0) * (a + i2));
        d = 1.0 + num * d;
        if (fabs(d) < tiny)
            d = tiny;
        c = 1.0 + num / c;
        if (fabs(c) < tiny)
            c = tiny;
        d = 1.0 / d;
        h *= d * c;
        num = -(a + i) * (a + b + i) * x / ((a + i2) * (a + i2 + 1.0));
        d = 1.0 + num * d;
        if (fabs(d) < tiny)
            d = tiny;
        c = 1.0 + num / c;
        if (fabs(c) < tiny)
            c = tiny;
        d = 1.0 / d;
        const double del = d * c;
        h *= del;
        if (fabs(del - 1.0) < 1e-16)
            break;
    }
    return h;
}

// I_x(a, b)
double reg_inc_beta(double a, double b, double x)
{
    if (x <= 0.0)
        return 0.0;
    if (x >= 1.0)
        return 1.0;
    const double front = exp(lgamma(a + b) - lgamma(a) - lgamma(b) + a * log(x) + b * log1p(-x));
    if (x < (a + 1.0) / (a + b + 2.0))
        return front * beta_cf(a, b, x) / a;
    return 1.0 - front * beta_cf(b, a, 1.0 - x) / b;
}

// P(|T| > t) for Student's t with df degrees of freedom
double t_two_sided_tail(double t, double df) { return reg_inc_beta(0.5 * df, 0.5, df / (df + t * t)); }

struct EstPlan {
    int64_t total; // sampled chunks over all tables
    size_t chunks_bytes, c_bytes;
};

bool est_plan(const fae_tables *tables, const int64_t *h_n_chunks, EstPlan *p)
{
    p->total = 0;
    for (int z = 0; z < tables->n_tables; ++z) {
        if (h_n_chunks[z] < 0)
            return false;
        p->total += h_n_chunks[z];
    }
    p->chunks_bytes = fae_align_up((size_t)(p->total + 1) * sizeof(int64_t), 256);
    p->c_bytes = fae_align_up((size_t)(p->total + 1) * sizeof(int32_t), 256);
    return p->total < (1 << 30);
}

// Everything a probe needs: validated arguments, the chunk numbers on the device.
struct Estimator {
    fae_ctx *ctx;
    const fae_tables *tables;
    const int64_t *h_n_chunks;
    int64_t m;
    EstArgs a;
    EstPlan plan;
    std::vector<int32_t> C;  // host copy of the counts of the last probe
    std::vector<int64_t> N;  // chunks per table

    int32_t setup(fae_ctx *c, const fae_tables *t, const uint32_t *const *h_counts, int64_t m_, const int64_t *n_chunks,
                  const int64_t *const *h_chunks, void *ws, size_t ws_bytes, const char *who)
    {
        ctx = c;
        tables = t;
        h_n_chunks = n_chunks;
        m = m_;
        int32_t rc = fae_check_tables(ctx, tables, who);
        if (rc != FAE_OK)
            return rc;
        if (!h_counts || !n_chunks || !h_chunks || m <= 0)
            return fae_fail(ctx, FAE_EINVAL, "%s: null argument or m <= 0", who);
        if (!est_plan(tables, n_chunks, &plan))
            return fae_fail(ctx, FAE_EINVAL, "%s: bad number of chunks", who);
        if (!ws || ws_bytes < plan.chunks_bytes + plan.c_bytes)
            return fae_fail(ctx, FAE_ENOSPC, "%s: workspace too small", who);
        const int nt = tables->n_tables;
        memset(&a, 0, sizeof(a));
        N.assign(nt, 0);
        std::vector<int64_t> all;
        all.reserve((size_t)plan.total + 1);
        int64_t start = 0;
        for (int z = 0; z < nt; ++z) {
            N[z] = (tables->h_rows[z] + m - 1) / m;
            a.counts[z] = h_counts[z];
            a.rows[z] = tables->h_rows[z];
            a.chunk_start[z] = (int32_t)start;
            if (n_chunks[z] > N[z])
                return fae_fail(ctx, FAE_EINVAL, "%s: table %d has %lld chunks, %lld asked for", who, z,
                                (long long)N[z], (long long)n_chunks[z]);
            if (n_chunks[z] > 0 && (!h_chunks[z] || !h_counts[z]))
                return fae_fail(ctx, FAE_EINVAL, "%s: null pointer for table %d", who, z);
            std::vector<int64_t> seen(h_chunks[z], h_chunks[z] + n_chunks[z]);
            std::sort(seen.begin(), seen.end());
            for (size_t i = 0; i < seen.size(); ++i)
                if (seen[i] < 0 || seen[i] >= N[z] || (i > 0 && seen[i] == seen[i - 1]))
                    return fae_fail(ctx, FAE_EINVAL, "%s: chunk numbers of table %d must be distinct and inside [0, %lld)",
                                    who, z, (long long)N[z]);
            all.insert(all.end(), h_chunks[z], h_chunks[z] + n_chunks[z]);
            start += n_chunks[z];
        }
        a.chunk_start[nt] = (int32_t)start;
        a.chunks = (const int64_t *)ws;
        a.C = (int32_t *)((char *)ws + plan.chunks_bytes);
        a.m = m;
        a.n_tables = nt;
        C.assign((size_t)plan.total + 1, 0);
        FAE_HIP(ctx, hipSetDevice(ctx->device));
        if (plan.total > 0) {
            FAE_HIP(ctx, hipMemcpyAsync((void *)a.chunks, all.data(), (size_t)plan.total * sizeof(int64_t),
                                        hipMemcpyHostToDevice, ctx->stream));
            FAE_HIP(ctx, hipStreamSynchronize(ctx->stream)); // `all` goes out of scope
        }
        return FAE_OK;
    }

    // C_i of every sampled chunk at the cutoffs H[z] (Eq. 2), on the host afterwards
    int32_t probe(const uint32_t *H)
    {
        if (plan.total == 0)
            return FAE_OK;
        for (int z = 0; z < tables->n_tables; ++z)
            a.cutoff[z] = H[z];
        {
            fae_ktimer kt(ctx, FAE_K_ESTIMATE);
            FAE_LAUNCH(ctx, est_chunk_count_kernel, dim3((unsigned)plan.total), dim3(EST_THREADS), 0, ctx->stream, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        FAE_HIP(ctx, hipMemcpyAsync(C.data(), a.C, (size_t)plan.total * sizeof(int32_t), hipMemcpyDeviceToHost,
                                    ctx->stream));
        FAE_HIP(ctx, hipStreamSynchronize(ctx->stream));
        return FAE_OK;
    }

    int64_t sum_C(int z) const
    {
        int64_t s = 0;
        for (int i = a.chunk_start[z]; i < a.chunk_start[z + 1]; ++i)
            s += C[(size_t)i];
        return s;
    }

    // Eq. 3 and Eq. 4 for table z from the counts of the last probe
    void stats(int z, double t_quantile, fae_hot_estimate *e) const
    {
        const int64_t n = h_n_chunks[z];
        e->N = N[z];
        e->n = n;
        e->rows = e->half_rows = e->ybar = e->s = 0.0;
        if (n == 0)
            return;
        e->ybar = (double)sum_C(z) / (double)n;
        double ss = 0.0;
        for (int i = a.chunk_start[z]; i < a.chunk_start[z + 1]; ++i) {
            const double d = (double)C[(size_t)i] - e->ybar;
            ss += d * d;
        }
        e->s = n > 1 ? sqrt(ss / (double)(n - 1)) : 0.0;
        const double half = t_quantile * sqrt(((double)(N[z] - n) / (double)N[z]) * (e->s * e->s / (double)n));
        e->rows = e->ybar * (double)N[z];
        e->half_rows = half * (double)N[z];
    }
};

inline uint64_t est_scaled_cutoff(uint64_t c, uint64_t T, uint64_t n)
{
    unsigned __int128 v = ((unsigned __int128)c * T + n - 1) / n;
    return v > 4294967295ull ? 4294967295ull : (uint64_t)v;
}
} // namespace

extern "C" double fae_t_quantile(double confidence, int64_t df)
{
    if (!(confidence > 0.0 && confidence < 1.0) || df < 1)
        return -1.0;
    const double alpha = 1.0 - confidence;
    double lo = 0.0, hi = 1.0;
    while (t_two_sided_tail(hi, (double)df) > alpha && hi < 1e300)
        hi *= 2.0;
    for (int i = 0; i < 200 && hi - lo > 1e-15 * hi; ++i) {
        const double mid = 0.5 * (lo + hi);
        if (t_two_sided_tail(mid, (double)df) > alpha)
            lo = mid;
        else
            hi = mid;
    }
    return 0.5 * (lo + hi);
}

extern "C" size_t fae_estimate_workspace_bytes(const fae_tables *tables, const int64_t *h_n_chunks)
{
    EstPlan p;
    if (!tables || !h_n_chunks || tables->n_tables < 1 || tables->n_tables > FAE_MAX_TABLES ||
        !est_plan(tables, h_n_chunks, &p))
        return 0;
    return p.chunks_bytes + p.c_bytes;
}

extern "C" int32_t fae_estimate_hot(fae_ctx *ctx, const fae_tables *tables, const uint32_t *const *h_counts,
                                    const uint32_t *h_cutoff, int64_t m, const int64_t *h_n_chunks,
                                    const int64_t *const *h_chunks, double confidence, fae_hot_estimate *h_out,
                                    int32_t *h_C_out, void *ws, size_t ws_bytes)
{
    if (!ctx)
        return FAE_EINVAL;
    if (!h_cutoff || !h_out || !(confidence > 0.0 && confidence < 1.0))
        return fae_fail(ctx, FAE_EINVAL, "fae_estimate_hot: null argument or confidence outside (0, 1)");
    Estimator est;
    int32_t rc = est.setup(ctx, tables, h_counts, m, h_n_chunks, h_chunks, ws, ws_bytes, "fae_estimate_hot");
    if (rc != FAE_OK)
        return rc;
    rc = est.probe(h_cutoff);
    if (rc != FAE_OK)
        return rc;
    for (int z = 0; z < tables->n_tables; ++z)
        est.stats(z, h_n_chunks[z] > 1 ? fae_t_quantile(confidence, h_n_chunks[z] - 1) : 0.0, &h_out[z]);
    if (h_C_out)
        for (int64_t i = 0; i < est.plan.total; ++i)
            h_C_out[i] = est.C[(size_t)i];
    return FAE_OK;
}

extern "C" int32_t fae_choose_cutoff_sampled(fae_ctx *ctx, const fae_tables *tables, const uint32_t *const *h_counts,
                                             const int64_t *h_T, int64_t t_denom, int64_t budget_bytes,
                                             int64_t small_table_bytes, int64_t m, const int64_t *h_n_chunks,
                                             const int64_t *const *h_chunks, double confidence, int64_t *h_c_out,
                                             uint32_t *h_cutoff_out, fae_hot_estimate *h_out, void *ws,
                                             size_t ws_bytes)
{
    if (!ctx)
        return FAE_EINVAL;
    if (!h_T || !h_c_out || !h_cutoff_out || !h_out || t_denom <= 0 || budget_bytes < 0 ||
        !(confidence > 0.0 && confidence < 1.0))
        return fae_fail(ctx, FAE_EINVAL, "fae_choose_cutoff_sampled: null or out-of-range argument");
    Estimator est;
    int32_t rc =
        est.setup(ctx, tables, h_counts, m, h_n_chunks, h_chunks, ws, ws_bytes, "fae_choose_cutoff_sampled");
    if (rc != FAE_OK)
        return rc;
    const int nt = tables->n_tables;
    const double row_bytes = (double)((int64_t)tables->dim * 4);
    bool small[FAE_MAX_TABLES];
    uint64_t max_T = 0;
    for (int z = 0; z < nt; ++z) {
        if (h_T[z] < 0)
            return fae_fail(ctx, FAE_EINVAL, "fae_choose_cutoff_sampled: negative T[%d]", z);
        small[z] = tables->h_rows[z] * (int64_t)tables->dim * 4 < small_table_bytes;
        if (!small[z] && h_n_chunks[z] < 1)
            return fae_fail(ctx, FAE_EINVAL, "fae_choose_cutoff_sampled: table %d is sampled but has no chunks", z);
        if (!small[z] && (uint64_t)h_T[z] > max_T)
            max_T = (uint64_t)h_T[z];
    }
    uint32_t H[FAE_MAX_TABLES];
    // estimated bytes of the hot set at threshold c
    auto bytes_at = [&](uint64_t c, double *bytes) -> int32_t {
        for (int z = 0; z < nt; ++z)
            H[z] = small[z] ? 0u : (uint32_t)est_scaled_cutoff(c, (uint64_t)h_T[z], (uint64_t)t_denom);
        int32_t r = est.probe(H);
        if (r != FAE_OK)
            return r;
        double b = 0.0;
        for (int z = 0; z < nt; ++z) {
            if (small[z])
                b += (double)tables->h_rows[z] * row_bytes;
            else
                b += ((double)est.sum_C(z) / (double)h_n_chunks[z]) * (double)est.N[z] * row_bytes;
        }
        *bytes = b;
        return FAE_OK;
    };
    auto finish = [&](uint64_t c) -> int32_t {
        double b;
        int32_t r = bytes_at(c, &b); // leaves the counts of c in est.C
        if (r != FAE_OK)
            return r;
        *h_c_out = (int64_t)c;
        for (int z = 0; z < nt; ++z) {
            h_cutoff_out[z] = H[z];
            est.stats(z, h_n_chunks[z] > 1 ? fae_t_quantile(confidence, h_n_chunks[z] - 1) : 0.0, &h_out[z]);
            if (small[z]) { // wholly hot, known exactly
                h_out[z].rows = (double)tables->h_rows[z];
                h_out[z].half_rows = 0.0;
            }
        }
        return FAE_OK;
    };
    double bytes;
    rc = bytes_at(0, &bytes);
    if (rc != FAE_OK)
        return rc;
    if (bytes <= (double)budget_bytes)
        return finish(0);
    // Beyond hi every sampled table's cutoff exceeds any 32-bit count it could hold, or T is 0
    // and the cutoff never moves; counts are < 2^32, so c = 2^32 * t_denom / T suffices.
    uint64_t lo = 0, hi = 1;
    for (;;) {
        rc = bytes_at(hi, &bytes);
        if (rc != FAE_OK)
            return rc;
        if (bytes <= (double)budget_bytes)
            break;
        bool saturated = true; // every movable cutoff already at the largest count value
        for (int z = 0; z < nt; ++z)
            saturated = saturated && (small[z] || h_T[z] == 0 || H[z] == 4294967295u);
        if (saturated || hi > (1ull << 62))
            return fae_fail(ctx, FAE_ENOSPC, "fae_choose_cutoff_sampled: no threshold fits the budget");
        lo = hi;
        hi *= 2;
    }
    while (hi - lo > 1) {
        const uint64_t mid = lo + (hi - lo) / 2;
        rc = bytes_at(mid, &bytes);
        if (rc != FAE_OK)
            return rc;
        if (bytes <= (double)budget_bytes)
            hi = mid;
        else
            lo = mid;
    }
    return finish(hi);
}
