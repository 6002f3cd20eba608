// Pre-processing stages on the GPU: Embedding Logger (access histogram), hot cutoff
// under a memory budget, Embedding Classifier (tag + remap + hot-id list) and
// Embedding Replicator (hot rows gathered into their own HBM-resident tables).
#include <stdlib.h>

#include <vector>

#include "fae_internal.h"

// =================================================================================
// a1  Embedding Logger: counts_z[r] += #lookups of r        (Sec. 4.1.2)
// =================================================================================
struct ProfArgs {
    const void *idx[FAE_MAX_TABLES]; // int32 or int64 row ids
    int32_t wide;                    // the ids are int64
    uint32_t *cnt[FAE_MAX_TABLES];
    int32_t n_rows[FAE_MAX_TABLES];
    int32_t n_lookups[FAE_MAX_TABLES];
    int32_t blk_start[FAE_MAX_TABLES + 1];
    int32_t n_tables;
    int32_t span; // lookups handled by one workgroup
    uint32_t *status;
};

// Baseline: one global atomic per lookup.
__global__ __launch_bounds__(256) void prof_atomic_kernel(ProfArgs a)
{
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int bl = blockIdx.x - a.blk_start[z];
    const void *idx = a.idx[z];
    uint32_t *cnt = a.cnt[z];
    const int n = a.n_lookups[z], R = a.n_rows[z];
    const int64_t beg = (int64_t)bl * a.span;
    const int64_t end = beg + a.span < n ? beg + a.span : n;
    bool bad = false;
    for (int64_t j = beg + threadIdx.x; j < end; j += 256) {
        const int r = fae_load_row(idx, j, a.wide, R);
        if (r >= 0)
            atomicAdd(&cnt[r], 1u);
        else
            bad = true;
    }
    if (bad)
        fae_flag(a.status, FAE_STATUS_ERANGE);
}

// LDS-privatised: a workgroup counts a long span of the stream in LDS and merges
// into the global counters once.  Small tables get a dense LDS copy of their
// counters; large tables a fixed-size LDS hash of the rows seen first (under a
// Zipf law the heavy hitters), anything that does not find a home goes straight
// to a global atomic.
#define PROF_THREADS 1024
#define PROF_DENSE_MAX 16384 // rows; 64 KiB of LDS counters
#define PROF_HASH_BITS 13
#define PROF_HASH_SIZE (1 << PROF_HASH_BITS)

__global__ __launch_bounds__(PROF_THREADS) void prof_lds_kernel(ProfArgs a)
{
    __shared__ uint32_t lds[PROF_DENSE_MAX]; // dense counters, or [keys | counts] of the hash
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int bl = blockIdx.x - a.blk_start[z];
    const void *idx = a.idx[z];
    uint32_t *cnt = a.cnt[z];
    const int n = a.n_lookups[z], R = a.n_rows[z];
    const int64_t beg = (int64_t)bl * a.span;
    const int64_t end = beg + a.span < n ? beg + a.span : n;
    bool bad = false;
    if (R <= PROF_DENSE_MAX) {
        for (int i = threadIdx.x; i < R; i += PROF_THREADS)
            lds[i] = 0u;
        __syncthreads();
        for (int64_t j = beg + threadIdx.x; j < end; j += PROF_THREADS) {
            const int r = fae_load_row(idx, j, a.wide, R);
            if (r >= 0)
                atomicAdd(&lds[r], 1u);
            else
                bad = true;
        }
        __syncthreads();
        for (int i = threadIdx.x; i < R; i += PROF_THREADS) {
            uint32_t c = lds[i];
            if (c)
                atomicAdd(&cnt[i], c);
        }
    } else {
        int32_t *keys = (int32_t *)lds;
        uint32_t *vals = lds + PROF_HASH_SIZE;
        for (int i = threadIdx.x; i < PROF_HASH_SIZE; i += PROF_THREADS) {
            keys[i] = -1;
            vals[i] = 0u;
        }
        __syncthreads();
        for (int64_t j = beg + threadIdx.x; j < end; j += PROF_THREADS) {
            const int r = fae_load_row(idx, j, a.wide, R);
            if (r < 0) {
                bad = true;
                continue;
            }
            uint32_t h = ((uint32_t)r * 2654435761u) >> (32 - PROF_HASH_BITS);
            bool done = false;
#pragma unroll
            for (int probe = 0; probe < 2 && !done; ++probe) {
                uint32_t slot = (h + probe) & (PROF_HASH_SIZE - 1);
                int old = atomicCAS(&keys[slot], -1, r);
                if (old == -1 || old == r) {
                    atomicAdd(&vals[slot], 1u);
                    done = true;
                }
            }
            if (!done)
                atomicAdd(&cnt[r], 1u);
        }
        __syncthreads();
        for (int i = threadIdx.x; i < PROF_HASH_SIZE; i += PROF_THREADS) {
            int k = keys[i];
            if (k >= 0)
                atomicAdd(&cnt[k], vals[i]);
        }
    }
    if (bad)
        fae_flag(a.status, FAE_STATUS_ERANGE);
}

extern "C" int32_t fae_profile(fae_ctx *ctx, const fae_tables *tables, const fae_batch *chunk,
                               uint32_t *const *h_counts)
{
    int32_t rc = fae_check_tables(ctx, tables, "fae_profile");
    if (rc != FAE_OK)
        return rc;
    rc = fae_check_batch(ctx, tables, chunk, "fae_profile");
    if (rc != FAE_OK)
        return rc;
    if (!h_counts)
        return fae_fail(ctx, FAE_EINVAL, "fae_profile: null counts");
    FAE_HIP(ctx, hipSetDevice(ctx->device));
    const int nt = tables->n_tables;
    const bool lds = ctx->opt_profile != 1;
    ProfArgs a;
    memset(&a, 0, sizeof(a));
    int64_t max_nl = 0;
    for (int z = 0; z < nt; ++z)
        if (chunk->h_n_lookups[z] > max_nl)
            max_nl = chunk->h_n_lookups[z];
    if (max_nl == 0)
        return FAE_OK;
    // a span long enough to aggregate duplicates in LDS, short enough to fill the chip
    int span = lds ? 65536 : 4096;
    if (lds) {
        while (span > 8192 && (max_nl / span) * nt < 2 * ctx->n_cu)
            span >>= 1;
    }
    a.span = span;
    int64_t blocks = 0;
    for (int z = 0; z < nt; ++z) {
        if (!h_counts[z] && tables->h_rows[z] > 0)
            return fae_fail(ctx, FAE_EINVAL, "fae_profile: null counters for table %d", z);
        a.idx[z] = chunk->h_indices[z];
        a.wide = chunk->index_bits == 64;
        a.cnt[z] = h_counts[z];
        a.n_rows[z] = (int32_t)tables->h_rows[z];
        a.n_lookups[z] = (int32_t)chunk->h_n_lookups[z];
        a.blk_start[z] = (int32_t)blocks;
        blocks += (chunk->h_n_lookups[z] + span - 1) / span;
    }
    a.blk_start[nt] = (int32_t)blocks;
    a.n_tables = nt;
    a.status = ctx->d_block;
    if (blocks >= 2147483647LL)
        return fae_fail(ctx, FAE_EINVAL, "fae_profile: chunk too large for one launch");
    fae_ktimer kt(ctx, FAE_K_PROFILE);
    if (lds)
        FAE_LAUNCH(ctx, prof_lds_kernel, dim3((unsigned)blocks), dim3(PROF_THREADS), 0, ctx->stream, a);
    else
        FAE_LAUNCH(ctx, prof_atomic_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, a);
    FAE_LAUNCH_CHECK(ctx);
    return FAE_OK;
}

// =================================================================================
// a2  hot cutoff: how many rows have count >= H, for a window of H values   (Eq. 2)
// =================================================================================
#define CW_BINS 2048
#define CW_TILE 8192 // rows per workgroup: 32 per thread, eight 16-byte loads
#define CW_STRIDE (CW_BINS + 2) // per table: bins, rows above the window, max count
#define CW_LOCAL 4 // the lowest bins of the window are counted in registers

struct CwArgs {
    const uint32_t *cnt[FAE_MAX_TABLES];
    int32_t n_rows[FAE_MAX_TABLES];
    uint32_t lo[FAE_MAX_TABLES];
    int32_t blk_start[FAE_MAX_TABLES + 1];
    int32_t n_tables;
    int32_t tiles_per_wg; // consecutive tiles of CW_TILE rows a workgroup counts before it merges
    uint32_t *hist; // [n_tables][CW_STRIDE], zeroed by the caller
};

// sum of v over the lanes of a wave (every lane gets it)
__device__ __forceinline__ uint32_t cw_wave_sum(uint32_t v)
{
#pragma unroll
    for (int m = 1; m < FAE_WAVE; m <<= 1)
        v += __shfl_xor(v, m, FAE_WAVE);
    return v;
}

// hist[z][b] = #rows with count == lo_z + b (b < CW_BINS); hist[z][CW_BINS] = #rows
// with count >= lo_z + CW_BINS; hist[z][CW_BINS+1] = max count.
// Under a skewed access law almost every row sits in the first bins of the window (never or once
// accessed), so one LDS counter per bin would have a whole wave hammering the same word: the
// CW_LOCAL lowest bins are counted in registers and added up per wave; the rest go to LDS.
__global__ __launch_bounds__(256) void count_window_kernel(CwArgs a)
{
    __shared__ uint32_t bins[CW_BINS + 2];
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int bl = blockIdx.x - a.blk_start[z];
    const uint32_t *cnt = a.cnt[z];
    const int R = a.n_rows[z];
    const uint32_t lo = a.lo[z];
    for (int i = threadIdx.x; i < CW_BINS + 2; i += 256)
        bins[i] = 0u;
    __syncthreads();
    uint32_t above = 0, mx = 0;
    uint32_t local[CW_LOCAL] = {0, 0, 0, 0};
    auto count = [&](uint32_t v) {
        mx = v > mx ? v : mx;
        if (v >= lo) {
            const uint32_t b = v - lo;
#pragma unroll
            for (int q = 0; q < CW_LOCAL; ++q)
                local[q] += b == (uint32_t)q ? 1u : 0u;
            if (b >= CW_BINS)
                above += 1;
            else if (b >= CW_LOCAL)
                atomicAdd(&bins[b], 1u);
        }
    };
    constexpr int VEC = CW_TILE / 256 / 4; // 16-byte loads per thread
    // several tiles per workgroup: the merge into the table's bins (the same few words for every
    // workgroup of a table) is paid once per workgroup, not once per tile
    for (int t = 0; t < a.tiles_per_wg; ++t) {
        const int64_t beg = ((int64_t)bl * a.tiles_per_wg + t) * CW_TILE;
        if (beg >= R)
            break;
        if (beg + CW_TILE <= R && (((uintptr_t)(cnt + beg)) & 15) == 0) {
            uint4 v[VEC];
#pragma unroll
            for (int k = 0; k < VEC; ++k) // every load is issued before the first is counted
                v[k] = ((const uint4 *)(cnt + beg))[k * 256 + threadIdx.x];
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                count(v[k].x);
                count(v[k].y);
                count(v[k].z);
                count(v[k].w);
            }
        } else {
            for (int k = 0; k < CW_TILE / 256; ++k) {
                const int64_t r = beg + k * 256 + threadIdx.x;
                if (r < R)
                    count(cnt[r]);
            }
        }
    }
#pragma unroll
    for (int q = 0; q < CW_LOCAL; ++q) {
        const uint32_t c = cw_wave_sum(local[q]);
        if (fae_lane() == 0 && c)
            atomicAdd(&bins[q], c);
    }
    above = cw_wave_sum(above);
    if (fae_lane() == 0 && above)
        atomicAdd(&bins[CW_BINS], above);
    if (mx)
        atomicMax(&bins[CW_BINS + 1], mx);
    __syncthreads();
    uint32_t *out = a.hist + (size_t)z * CW_STRIDE;
    for (int i = threadIdx.x; i < CW_BINS + 1; i += 256) {
        uint32_t c = bins[i];
        if (c)
            atomicAdd(&out[i], c);
    }
    if (threadIdx.x == 0 && bins[CW_BINS + 1])
        atomicMax(&out[CW_BINS + 1], bins[CW_BINS + 1]);
}

extern "C" size_t fae_choose_cutoff_workspace_bytes(const fae_tables *tables)
{
    if (!tables)
        return 0;
    return fae_align_up((size_t)FAE_MAX_TABLES * CW_STRIDE * sizeof(uint32_t), 256) + 256;
}

namespace {
struct Window {
    fae_ctx *ctx;
    const fae_tables *t;
    const uint32_t *const *h_counts;
    uint32_t *d_hist;
    std::vector<uint32_t> host; // [nt][CW_STRIDE]
    uint32_t lo[FAE_MAX_TABLES];

    int32_t run(const uint32_t *new_lo)
    {
        const int nt = t->n_tables;
        CwArgs a;
        memset(&a, 0, sizeof(a));
        int64_t blocks = 0, tiles = 0;
        for (int z = 0; z < nt; ++z)
            tiles += (t->h_rows[z] + CW_TILE - 1) / CW_TILE;
        // about eight workgroups per compute unit, each counting a run of consecutive tiles
        int64_t per = (tiles + 8LL * ctx->n_cu - 1) / (8LL * ctx->n_cu);
        if (per < 1)
            per = 1;
        a.tiles_per_wg = (int32_t)per;
        for (int z = 0; z < nt; ++z) {
            lo[z] = new_lo[z];
            a.cnt[z] = h_counts[z];
            a.n_rows[z] = (int32_t)t->h_rows[z];
            a.lo[z] = lo[z];
            a.blk_start[z] = (int32_t)blocks;
            blocks += ((t->h_rows[z] + CW_TILE - 1) / CW_TILE + per - 1) / per;
        }
        a.blk_start[nt] = (int32_t)blocks;
        a.n_tables = nt;
        a.hist = d_hist;
        int32_t rc = fae_fill_u32(ctx, d_hist, (int64_t)nt * CW_STRIDE, 0u);
        if (rc != FAE_OK)
            return rc;
        if (blocks > 0) {
            fae_ktimer kt(ctx, FAE_K_BUILD);
            FAE_LAUNCH(ctx, count_window_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        host.resize((size_t)nt * CW_STRIDE);
        FAE_HIP(ctx, hipMemcpyAsync(host.data(), d_hist, host.size() * sizeof(uint32_t), hipMemcpyDeviceToHost,
                                    ctx->stream));
        FAE_HIP(ctx, hipStreamSynchronize(ctx->stream));
        // bins -> suffix sums: host[z][b] = #rows with count >= lo_z + b
        for (int z = 0; z < nt; ++z) {
            uint32_t *h = &host[(size_t)z * CW_STRIDE];
            for (int b = CW_BINS - 1; b >= 0; --b)
                h[b] += h[b + 1];
        }
        return FAE_OK;
    }
    bool covers(int z, uint64_t H) const { return H >= lo[z] && H <= (uint64_t)lo[z] + CW_BINS; }
    // rows of table z with count >= H (H inside the window)
    int64_t n_hot(int z, uint64_t H) const
    {
        return (int64_t)host[(size_t)z * CW_STRIDE + (size_t)(H - lo[z])];
    }
    uint32_t max_count(int z) const { return host[(size_t)z * CW_STRIDE + CW_BINS + 1]; }
};

inline uint64_t scaled_cutoff(uint64_t c, uint64_t T, uint64_t n)
{
    unsigned __int128 v = ((unsigned __int128)c * T + n - 1) / n;
    return v > 4294967295ull ? 4294967295ull : (uint64_t)v;
}
} // namespace

extern "C" int32_t fae_count_hot(fae_ctx *ctx, const fae_tables *tables, const uint32_t *const *h_counts,
                                 const uint32_t *h_cutoff, int64_t *h_n_hot_out, void *ws, size_t ws_bytes)
{
    int32_t rc = fae_check_tables(ctx, tables, "fae_count_hot");
    if (rc != FAE_OK)
        return rc;
    if (!h_counts || !h_cutoff || !h_n_hot_out)
        return fae_fail(ctx, FAE_EINVAL, "fae_count_hot: null argument");
    if (!ws || ws_bytes < fae_choose_cutoff_workspace_bytes(tables))
        return fae_fail(ctx, FAE_ENOSPC, "fae_count_hot: workspace too small");
    FAE_HIP(ctx, hipSetDevice(ctx->device));
    Window w{ctx, tables, h_counts, (uint32_t *)ws, {}, {}};
    rc = w.run(h_cutoff);
    if (rc != FAE_OK)
        return rc;
    for (int z = 0; z < tables->n_tables; ++z)
        h_n_hot_out[z] = w.n_hot(z, h_cutoff[z]);
    return FAE_OK;
}

extern "C" int32_t fae_choose_cutoff(fae_ctx *ctx, const fae_tables *tables, const uint32_t *const *h_counts,
                                     const int64_t *h_T, int64_t t_denom, int64_t budget_bytes,
                                     int64_t small_table_bytes, int64_t *h_c_out, uint32_t *h_cutoff_out,
                                     int64_t *h_n_hot_out, void *ws, size_t ws_bytes)
{
    int32_t rc = fae_check_tables(ctx, tables, "fae_choose_cutoff");
    if (rc != FAE_OK)
        return rc;
    if (!h_counts || !h_T || !h_c_out || !h_cutoff_out || !h_n_hot_out || t_denom <= 0 || budget_bytes < 0)
        return fae_fail(ctx, FAE_EINVAL, "fae_choose_cutoff: null or non-positive argument");
    if (!ws || ws_bytes < fae_choose_cutoff_workspace_bytes(tables))
        return fae_fail(ctx, FAE_ENOSPC, "fae_choose_cutoff: workspace too small");
    FAE_HIP(ctx, hipSetDevice(ctx->device));
    const int nt = tables->n_tables;
    const int64_t row_bytes = (int64_t)tables->dim * 4;
    bool small[FAE_MAX_TABLES];
    for (int z = 0; z < nt; ++z) {
        if (h_T[z] < 0)
            return fae_fail(ctx, FAE_EINVAL, "fae_choose_cutoff: negative T[%d]", z);
        small[z] = tables->h_rows[z] * row_bytes < small_table_bytes;
    }
    auto H_of = [&](int z, uint64_t c) -> uint64_t {
        return small[z] ? 0ull : scaled_cutoff(c, (uint64_t)h_T[z], (uint64_t)t_denom);
    };
    Window w{ctx, tables, h_counts, (uint32_t *)ws, {}, {}};
    uint32_t lo0[FAE_MAX_TABLES] = {0};
    rc = w.run(lo0);
    if (rc != FAE_OK)
        return rc;
    uint32_t maxc[FAE_MAX_TABLES];
    for (int z = 0; z < nt; ++z)
        maxc[z] = w.max_count(z);
    // evaluate(c): total bytes of hot rows at threshold c, if every H_z(c) is inside the window
    auto evaluate = [&](uint64_t c, int64_t *bytes) -> bool {
        int64_t b = 0;
        for (int z = 0; z < nt; ++z) {
            uint64_t H = H_of(z, c);
            if (!w.covers(z, H))
                return false;
            b += w.n_hot(z, H) * row_bytes;
        }
        *bytes = b;
        return true;
    };
    auto finish = [&](uint64_t c) -> int32_t {
        *h_c_out = (int64_t)c;
        for (int z = 0; z < nt; ++z) {
            uint64_t H = H_of(z, c);
            h_cutoff_out[z] = (uint32_t)H;
            h_n_hot_out[z] = w.n_hot(z, H);
        }
        return FAE_OK;
    };
    bool any_scalable = false;
    for (int z = 0; z < nt; ++z)
        any_scalable = any_scalable || (!small[z] && h_T[z] > 0);
    if (!any_scalable) { // no cutoff moves with c: either everything fits or nothing will
        int64_t b0 = 0;
        (void)evaluate(0, &b0);
        if (b0 <= budget_bytes)
            return finish(0);
        return fae_fail(ctx, FAE_ENOSPC, "fae_choose_cutoff: the wholly-hot tables alone exceed the budget");
    }
    // phase 1: walk c upward inside the first window (the common case: small cutoffs)
    uint64_t c = 0;
    int64_t bytes = 0;
    while (evaluate(c, &bytes)) {
        if (bytes <= budget_bytes)
            return finish(c);
        ++c;
    }
    // phase 2: the answer lies beyond the first window; bisect on c, one window per probe
    uint64_t lo_c = c - 1; // known not to fit (c >= 1 here: c = 0 is always inside the first window)
    uint64_t hi_c = 1;
    for (int z = 0; z < nt; ++z) {
        if (small[z] || h_T[z] == 0)
            continue;
        // smallest c with H_z(c) > maxc[z]
        unsigned __int128 need = ((unsigned __int128)(maxc[z] + 1ull) * (uint64_t)t_denom + h_T[z] - 1) /
                                 (uint64_t)h_T[z];
        uint64_t cz = (uint64_t)need + 1;
        if (cz > hi_c)
            hi_c = cz;
    }
    auto probe = [&](uint64_t cc, int64_t *b) -> int32_t {
        uint32_t lo[FAE_MAX_TABLES];
        for (int z = 0; z < nt; ++z)
            lo[z] = (uint32_t)H_of(z, cc);
        int32_t r = w.run(lo);
        if (r != FAE_OK)
            return r;
        return evaluate(cc, b) ? FAE_OK : fae_fail(ctx, FAE_EINVAL, "fae_choose_cutoff: internal window error");
    };
    if (hi_c <= lo_c)
        hi_c = lo_c + 1;
    rc = probe(hi_c, &bytes);
    if (rc != FAE_OK)
        return rc;
    if (bytes > budget_bytes)
        return fae_fail(ctx, FAE_ENOSPC, "fae_choose_cutoff: the wholly-hot small tables alone exceed the budget");
    while (hi_c - lo_c > 1) {
        uint64_t mid = lo_c + (hi_c - lo_c) / 2;
        rc = probe(mid, &bytes);
        if (rc != FAE_OK)
            return rc;
        if (bytes <= budget_bytes)
            hi_c = mid;
        else
            lo_c = mid;
    }
    rc = probe(hi_c, &bytes);
    if (rc != FAE_OK)
        return rc;
    return finish(hi_c);
}

// =================================================================================
// a3  Embedding Classifier: tag, remap, hot-id list               (Sec. 4.2, Eq. 2)
// =================================================================================
#define BT_TILE 2048 // rows per workgroup (8 per thread, contiguous)

struct BuildArgs {
    const uint32_t *cnt[FAE_MAX_TABLES];
    int32_t *remap[FAE_MAX_TABLES];
    int32_t *hot_ids[FAE_MAX_TABLES];
    int32_t n_rows[FAE_MAX_TABLES];
    uint32_t cutoff[FAE_MAX_TABLES];
    int32_t cap[FAE_MAX_TABLES];
    int32_t tile_start[FAE_MAX_TABLES + 1];
    int32_t n_tables;
    int32_t *tile_sums; // [total_tiles + 1]
    uint32_t *status;
    uint32_t *n_hot_out; // device scalars, one per table
};

__device__ __forceinline__ void build_load8(const uint32_t *cnt, int64_t r0, int R, uint32_t v[8])
{
    if (r0 + 8 <= R && (((uintptr_t)(cnt + r0)) & 15) == 0) {
        uint4 a = *(const uint4 *)(cnt + r0);
        uint4 b = *(const uint4 *)(cnt + r0 + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k)
            v[k] = (r0 + k < R) ? cnt[r0 + k] : 0u;
    }
}

__global__ __launch_bounds__(256) void build_count_kernel(BuildArgs a)
{
    __shared__ int lds[256 / FAE_WAVE + 1];
    const int z = fae_find_table(a.tile_start, a.n_tables, blockIdx.x);
    const int tl = blockIdx.x - a.tile_start[z];
    const int R = a.n_rows[z];
    const uint32_t H = a.cutoff[z];
    const int64_t r0 = (int64_t)tl * BT_TILE + (int64_t)threadIdx.x * 8;
    uint32_t v[8];
    build_load8(a.cnt[z], r0, R, v);
    int c = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k)
        c += (r0 + k < R && v[k] >= H) ? 1 : 0;
    int total;
    (void)fae_block_excl_scan<256>(c, lds, &total);
    if (threadIdx.x == 0)
        a.tile_sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void build_scatter_kernel(BuildArgs a)
{
    __shared__ int lds[256 / FAE_WAVE + 1];
    const int z = fae_find_table(a.tile_start, a.n_tables, blockIdx.x);
    const int tl = blockIdx.x - a.tile_start[z];
    const int R = a.n_rows[z];
    const uint32_t H = a.cutoff[z];
    const int cap = a.cap[z];
    const int64_t r0 = (int64_t)tl * BT_TILE + (int64_t)threadIdx.x * 8;
    uint32_t v[8];
    build_load8(a.cnt[z], r0, R, v);
    int c = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k)
        c += (r0 + k < R && v[k] >= H) ? 1 : 0;
    int total;
    int ex = fae_block_excl_scan<256>(c, lds, &total);
    // slots restart at 0 for every table: subtract the scan value at the table's first tile
    int slot = a.tile_sums[blockIdx.x] - a.tile_sums[a.tile_start[z]] + ex;
    int32_t *remap = a.remap[z];
    int32_t *hot_ids = a.hot_ids[z];
    bool over = false;
    int32_t rm[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        rm[k] = -1;
        if (r0 + k < R && v[k] >= H) {
            rm[k] = slot;
            if (slot < cap)
                hot_ids[slot] = (int32_t)(r0 + k);
            else
                over = true;
            ++slot;
        }
    }
    if (r0 + 8 <= R && (((uintptr_t)(remap + r0)) & 15) == 0) { // the eight entries as two 16-byte stores
        *(int4 *)(remap + r0) = make_int4(rm[0], rm[1], rm[2], rm[3]);
        *(int4 *)(remap + r0 + 4) = make_int4(rm[4], rm[5], rm[6], rm[7]);
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (r0 + k < R)
                remap[r0 + k] = rm[k];
    }
    if (over)
        fae_flag(a.status, FAE_STATUS_ENOSPC);
    if (tl == 0 && threadIdx.x == 0)
        a.n_hot_out[z] = (uint32_t)(a.tile_sums[a.tile_start[z + 1]] - a.tile_sums[a.tile_start[z]]);
}

// =================================================================================
// a4  Embedding Replicator: hot rows into their own table            (Sec. 4)
// =================================================================================
struct GatherArgs {
    const float *W[FAE_MAX_TABLES];
    float *hotW[FAE_MAX_TABLES];
    const int32_t *hot_ids[FAE_MAX_TABLES];
    int32_t n_hot[FAE_MAX_TABLES];
    int64_t blk_start[FAE_MAX_TABLES + 1];
    int32_t n_tables;
    int32_t dim;
    int32_t procedural;
    uint64_t seed;
};

__device__ __forceinline__ uint64_t dev_mix64(uint64_t x)
{
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

// Initial weight of element (row, col) of virtual table z: the top 24 bits of a
// 64-bit mix of a per-table key and the element counter, mapped to U(-0.05, 0.05).
__device__ __forceinline__ float dev_w0(uint64_t table_key, int64_t row, int dim, int col)
{
    uint64_t ctr = (uint64_t)row * (uint64_t)dim + (uint64_t)col + 1ull;
    uint64_t h = dev_mix64(table_key + 0xD1B54A32D192ED03ull * ctr);
    float u = (float)(uint32_t)(h >> 40);
    return (u * 0x1p-24f - 0.5f) * 0.1f;
}

template <typename V> __global__ __launch_bounds__(256) void gather_rows_kernel(GatherArgs a)
{
    constexpr int VW = sizeof(V) / sizeof(float);
    // blockIdx.x spans all tables; the prefix is 64-bit because a 64 GiB hot set has > 2^31 vectors
    int z = 0;
    const int64_t b = blockIdx.x;
    while (z + 1 < a.n_tables && b >= a.blk_start[z + 1])
        ++z;
    const int ncols = a.dim / VW;
    const int64_t e = (b - a.blk_start[z]) * 256 + threadIdx.x;
    const int64_t slot = e / ncols;
    const int c = (int)(e - slot * ncols);
    if (slot >= a.n_hot[z])
        return;
    const int64_t row = a.hot_ids[z][slot];
    V *dst = (V *)a.hotW[z] + slot * ncols + c;
    if (a.procedural) {
        const uint64_t key = dev_mix64(a.seed ^ (0x9E3779B97F4A7C15ull * (uint64_t)(z + 1)));
        float t[VW];
#pragma unroll
        for (int k = 0; k < VW; ++k)
            t[k] = dev_w0(key, row, a.dim, c * VW + k);
        *dst = *(V *)t;
    } else {
        *dst = ((const V *)a.W[z])[row * ncols + c];
    }
}

extern "C" size_t fae_build_workspace_bytes(const fae_tables *tables)
{
    if (!tables || !tables->h_rows)
        return 0;
    size_t tiles = 0;
    for (int z = 0; z < tables->n_tables; ++z)
        tiles += (size_t)((tables->h_rows[z] + BT_TILE - 1) / BT_TILE);
    return fae_align_up((tiles + 2) * sizeof(int32_t), 256) + 256;
}

extern "C" int32_t fae_build_hot_tables(fae_ctx *ctx, const fae_tables *tables, const uint32_t *const *h_counts,
                                        const uint32_t *h_cutoff, const fae_weight_src *src,
                                        int32_t *const *h_remap, int32_t *const *h_hot_ids,
                                        float *const *h_hotW, const int64_t *h_cap, int64_t *h_n_hot_out,
                                        void *ws, size_t ws_bytes)
{
    int32_t rc = fae_check_tables(ctx, tables, "fae_build_hot_tables");
    if (rc != FAE_OK)
        return rc;
    if (!h_counts || !h_cutoff || !src || !h_remap || !h_hot_ids || !h_hotW || !h_cap || !h_n_hot_out)
        return fae_fail(ctx, FAE_EINVAL, "fae_build_hot_tables: null argument");
    if (src->kind != FAE_SRC_DEVICE && src->kind != FAE_SRC_PROCEDURAL)
        return fae_fail(ctx, FAE_EINVAL, "fae_build_hot_tables: unknown weight source %d", src->kind);
    if (src->kind == FAE_SRC_DEVICE && !src->h_W)
        return fae_fail(ctx, FAE_EINVAL, "fae_build_hot_tables: FAE_SRC_DEVICE without table pointers");
    if (!ws || ws_bytes < fae_build_workspace_bytes(tables))
        return fae_fail(ctx, FAE_ENOSPC, "fae_build_hot_tables: workspace too small");
    FAE_HIP(ctx, hipSetDevice(ctx->device));
    const int nt = tables->n_tables, dim = tables->dim;
    BuildArgs a;
    memset(&a, 0, sizeof(a));
    int64_t tiles = 0;
    for (int z = 0; z < nt; ++z) {
        const int64_t R = tables->h_rows[z];
        if (h_cap[z] < 0)
            return fae_fail(ctx, FAE_EINVAL, "fae_build_hot_tables: negative capacity for table %d", z);
        if (R > 0 && (!h_counts[z] || !h_remap[z]))
            return fae_fail(ctx, FAE_EINVAL, "fae_build_hot_tables: null counters/remap for table %d", z);
        if (h_cap[z] > 0 && (!h_hot_ids[z] || !h_hotW[z]))
            return fae_fail(ctx, FAE_EINVAL, "fae_build_hot_tables: null hot_ids/hotW for table %d", z);
        if (src->kind == FAE_SRC_DEVICE && R > 0 && !src->h_W[z])
            return fae_fail(ctx, FAE_EINVAL, "fae_build_hot_tables: null source table %d", z);
        a.cnt[z] = h_counts[z];
        a.remap[z] = h_remap[z];
        a.hot_ids[z] = h_hot_ids[z];
        a.n_rows[z] = (int32_t)R;
        a.cutoff[z] = h_cutoff[z];
        a.cap[z] = (int32_t)(h_cap[z] > 2147483647LL ? 2147483647LL : h_cap[z]);
        a.tile_start[z] = (int32_t)tiles;
        tiles += (R + BT_TILE - 1) / BT_TILE;
    }
    a.tile_start[nt] = (int32_t)tiles;
    a.n_tables = nt;
    a.tile_sums = (int32_t *)ws;
    a.status = ctx->d_block;
    a.n_hot_out = ctx->d_block + FAE_BLK_SCALARS;
    if (tiles >= 2147483647LL)
        return fae_fail(ctx, FAE_EINVAL, "fae_build_hot_tables: too many rows for one launch");
    rc = fae_fill_u32(ctx, ctx->d_block + FAE_BLK_SCALARS, nt, 0u);
    if (rc != FAE_OK)
        return rc;
    if (tiles > 0) {
        fae_ktimer kt(ctx, FAE_K_BUILD);
        FAE_LAUNCH(ctx, build_count_kernel, dim3((unsigned)tiles), dim3(256), 0, ctx->stream, a);
        FAE_LAUNCH_CHECK(ctx);
    }
    rc = fae_scan_i32(ctx, a.tile_sums, tiles);
    if (rc != FAE_OK)
        return rc;
    if (tiles > 0) {
        fae_ktimer kt(ctx, FAE_K_BUILD);
        FAE_LAUNCH(ctx, build_scatter_kernel, dim3((unsigned)tiles), dim3(256), 0, ctx->stream, a);
        FAE_LAUNCH_CHECK(ctx);
    }
    rc = fae_readback(ctx, FAE_BLK_SCALARS, nt);
    if (rc != FAE_OK)
        return rc;
    for (int z = 0; z < nt; ++z)
        h_n_hot_out[z] = (int64_t)ctx->h_block[FAE_BLK_SCALARS + z];
    rc = fae_sync_status(ctx);
    if (rc != FAE_OK)
        return rc; // capacity overflow: hot_ids are incomplete, do not gather

    // gather (or generate) the hot rows
    GatherArgs g;
    memset(&g, 0, sizeof(g));
    bool vec = dim % 4 == 0;
    for (int z = 0; z < nt; ++z) {
        if (((uintptr_t)h_hotW[z]) % 16 != 0)
            vec = false;
        if (src->kind == FAE_SRC_DEVICE && ((uintptr_t)src->h_W[z]) % 16 != 0)
            vec = false;
    }
    const int ncols = vec ? dim / 4 : dim;
    int64_t blocks = 0;
    for (int z = 0; z < nt; ++z) {
        g.W[z] = src->kind == FAE_SRC_DEVICE ? src->h_W[z] : nullptr;
        g.hotW[z] = h_hotW[z];
        g.hot_ids[z] = h_hot_ids[z];
        g.n_hot[z] = (int32_t)h_n_hot_out[z];
        g.blk_start[z] = blocks;
        blocks += (h_n_hot_out[z] * ncols + 255) / 256;
    }
    g.blk_start[nt] = blocks;
    g.n_tables = nt;
    g.dim = dim;
    g.procedural = src->kind == FAE_SRC_PROCEDURAL;
    g.seed = src->seed;
    if (blocks >= 2147483647LL)
        return fae_fail(ctx, FAE_EINVAL, "fae_build_hot_tables: hot set too large for one launch");
    if (blocks > 0) {
        fae_ktimer kt(ctx, FAE_K_BUILD);
        if (vec)
            FAE_LAUNCH(ctx, gather_rows_kernel<float4>, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, g);
        else
            FAE_LAUNCH(ctx, gather_rows_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, g);
        FAE_LAUNCH_CHECK(ctx);
    }
    FAE_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return FAE_OK;
}
