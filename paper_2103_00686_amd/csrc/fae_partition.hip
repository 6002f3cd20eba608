// Input Classifier (Sec. 4.2): a sparse input is hot iff every access in every table
// hits a hot row.  Hot and cold inputs keep their original order; for the hot ones
// the hot slots and a rebuilt CSR are emitted so that consecutive slices are the
// hot mini-batches.  Integer-only work: random 4-byte gathers into the remap, an
// AND-reduction per sample, a stable compaction.
#include "fae_internal.h"

#define PT_TILE 1024 // samples per scan tile (4 per thread)

struct PartArgs {
    const void *idx[FAE_MAX_TABLES]; // int32 or int64 row ids
    int32_t wide;                    // the ids are int64
    const int32_t *offsets[FAE_MAX_TABLES];
    const int32_t *remap[FAE_MAX_TABLES];
    int32_t *slots[FAE_MAX_TABLES];
    int32_t *hoffsets[FAE_MAX_TABLES];
    int32_t n_rows[FAE_MAX_TABLES];
    int32_t n_lookups[FAE_MAX_TABLES];
    int32_t blk_start[FAE_MAX_TABLES + 1]; // lookup-parallel kernels: blocks of PT_BLOCK lookups
    int32_t n_tables;
    int32_t n_samples;
    int32_t n_tiles;      // sample tiles
    uint32_t *cold;       // [n_samples] 1 = some access is cold
    int32_t *hidx;        // [n_samples] position among hot samples
    int32_t *tile_sums;   // [(n_tables+1) * n_tiles + 1]; row 0 = hot flags, row z+1 = hot lookups of table z
    int32_t *hot_samples;
    int32_t *cold_samples;
    uint32_t *status;
    uint32_t *scalars;    // device scalars: [0] = n_hot_samples, [1+z] = hot lookups of table z
};

#define PT_LK 4                 // lookups per thread in the lookup-parallel kernels
#define PT_BLOCK (256 * PT_LK)  // lookups per workgroup there

// pass 1: mark samples with a cold (or invalid) access; PT_LK lookups per thread, a workgroup's
// loads of one round next to each other.  All index loads go out first, then all remap gathers.
__global__ __launch_bounds__(256) void part_mark_kernel(PartArgs a)
{
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int base = (blockIdx.x - a.blk_start[z]) * PT_BLOCK + threadIdx.x;
    const int nl = a.n_lookups[z];
    const int32_t *off = a.offsets[z];
    const int32_t *remap = a.remap[z];
    int r[PT_LK], s[PT_LK], m[PT_LK];
#pragma unroll
    for (int k = 0; k < PT_LK; ++k) {
        const int j = base + k * 256;
        r[k] = j < nl ? fae_load_row(a.idx[z], j, a.wide, a.n_rows[z]) : -2;
    }
#pragma unroll
    for (int k = 0; k < PT_LK; ++k) {
        const int j = base + k * 256;
        s[k] = (off && j < nl) ? fae_sample_of(off, a.n_samples, j) : j;
    }
#pragma unroll
    for (int k = 0; k < PT_LK; ++k)
        m[k] = r[k] >= 0 ? remap[r[k]] : -1;
#pragma unroll
    for (int k = 0; k < PT_LK; ++k) {
        if (r[k] == -2)
            continue;
        if (r[k] < 0)
            fae_flag(a.status, FAE_STATUS_ERANGE);
        if (m[k] < 0)
            a.cold[s[k]] = 1u; // benign race: every writer stores the same value
    }
}

__device__ __forceinline__ int part_len(const PartArgs &a, int z, int s, bool *bad)
{
    const int32_t *off = a.offsets[z];
    if (!off)
        return 1;
    int b = off[s], e = off[s + 1];
    if (b < 0 || e < b || e > a.n_lookups[z] || (s == 0 && b != 0) || (s == a.n_samples - 1 && e != a.n_lookups[z])) {
        *bad = true;
        return 0;
    }
    return e - b;
}

// pass 2: per tile of samples and per row (0: hot flag, z+1: hot lookups of table z) the tile total.
// Rows z+1 also validate the CSR of table z for every sample, hot or cold.
__global__ __launch_bounds__(256) void part_count_kernel(PartArgs a)
{
    __shared__ int lds[256 / FAE_WAVE + 1];
    const int tile = blockIdx.x, row = blockIdx.y;
    int c = 0;
    bool bad = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int s = tile * PT_TILE + threadIdx.x * 4 + k;
        if (s < a.n_samples) {
            int len = row == 0 ? 1 : part_len(a, row - 1, s, &bad);
            if (!a.cold[s])
                c += len;
        }
    }
    if (bad)
        fae_flag(a.status, FAE_STATUS_ERANGE);
    int total;
    (void)fae_block_excl_scan<256>(c, lds, &total);
    if (threadIdx.x == 0)
        a.tile_sums[row * a.n_tiles + tile] = total;
}

// pass 3 (after the scan of tile_sums): hot / cold sample lists and each sample's hot position;
// for the tables with one lookup per sample also the rebuilt offsets (hot sample h starts at h)
__global__ __launch_bounds__(256) void part_emit_kernel(PartArgs a)
{
    __shared__ int lds[256 / FAE_WAVE + 1];
    const int tile = blockIdx.x;
    int c = 0;
    uint32_t cold[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int s = tile * PT_TILE + threadIdx.x * 4 + k;
        cold[k] = s < a.n_samples ? a.cold[s] : 1u;
        c += cold[k] ? 0 : 1;
    }
    int total;
    int ex = fae_block_excl_scan<256>(c, lds, &total);
    const int run0 = a.tile_sums[tile] + ex; // row 0 starts the scanned array: its base is 0
    int run = run0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int s = tile * PT_TILE + threadIdx.x * 4 + k;
        if (s >= a.n_samples)
            break;
        if (!cold[k]) {
            a.hot_samples[run] = s;
            a.hidx[s] = run;
            ++run;
        } else {
            a.cold_samples[s - run] = s; // run = number of hot samples before s
            a.hidx[s] = -1;
        }
    }
    if (c > 0)
        for (int z = 0; z < a.n_tables; ++z) {
            if (a.offsets[z])
                continue;
            int32_t *hoff = a.hoffsets[z];
            for (int h = run0; h < run; ++h)
                hoff[h] = h;
        }
}

// pass 3b: hoffsets_z[h] for every hot sample (needs hidx from pass 3, row 0)
__global__ __launch_bounds__(256) void part_offsets_kernel(PartArgs a)
{
    __shared__ int lds[256 / FAE_WAVE + 1];
    const int tile = blockIdx.x, z = blockIdx.y;
    const int row = z + 1;
    const int row_base = a.tile_sums[row * a.n_tiles];
    int32_t *hoff = a.hoffsets[z];
    if (a.offsets[z]) { // one lookup per sample otherwise: pass 3 has written those offsets
        int v[4];
        int c = 0;
        bool bad = false;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            int s = tile * PT_TILE + threadIdx.x * 4 + k;
            v[k] = 0;
            if (s < a.n_samples && !a.cold[s])
                v[k] = part_len(a, z, s, &bad);
            c += v[k];
        }
        int total;
        int ex = fae_block_excl_scan<256>(c, lds, &total);
        int run = a.tile_sums[row * a.n_tiles + tile] - row_base + ex;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            int s = tile * PT_TILE + threadIdx.x * 4 + k;
            if (s >= a.n_samples)
                break;
            if (!a.cold[s])
                hoff[a.hidx[s]] = run;
            run += v[k];
        }
    }
    if (tile == 0 && threadIdx.x == 0) {
        // totals: hot samples and hot lookups of this table; closing offset
        const int n_hot = a.tile_sums[1 * a.n_tiles] - a.tile_sums[0];
        const int row_end = a.tile_sums[(row + 1) * a.n_tiles]; // first entry of the next row (or the grand total)
        hoff[n_hot] = row_end - row_base;
        a.scalars[1 + z] = (uint32_t)(row_end - row_base);
        if (z == 0)
            a.scalars[0] = (uint32_t)n_hot;
    }
}

// pass 4: hot slots of the hot samples' lookups, PT_LK input lookups per thread; loads of the same
// kind go out together
__global__ __launch_bounds__(256) void part_slots_kernel(PartArgs a)
{
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int base = (blockIdx.x - a.blk_start[z]) * PT_BLOCK + threadIdx.x;
    const int nl = a.n_lookups[z];
    const int32_t *off = a.offsets[z];
    const int32_t *remap = a.remap[z];
    const int32_t *hoff = a.hoffsets[z];
    int s[PT_LK], h[PT_LK], r[PT_LK], dst[PT_LK], m[PT_LK];
#pragma unroll
    for (int k = 0; k < PT_LK; ++k) {
        const int j = base + k * 256;
        s[k] = j < nl ? (off ? fae_sample_of(off, a.n_samples, j) : j) : -1;
    }
#pragma unroll
    for (int k = 0; k < PT_LK; ++k)
        h[k] = s[k] >= 0 ? a.hidx[s[k]] : -1; // -1 for a cold sample
#pragma unroll
    for (int k = 0; k < PT_LK; ++k) {
        const int j = base + k * 256;
        r[k] = h[k] >= 0 ? fae_load_row(a.idx[z], j, a.wide, a.n_rows[z]) : -1;
        dst[k] = -1;
        if (h[k] >= 0) {
            const int within = off ? j - off[s[k]] : 0;
            const int d = (off ? hoff[h[k]] : h[k]) + within;
            if (within >= 0 && d >= 0 && d < nl) // else: malformed CSR (already flagged)
                dst[k] = d;
        }
    }
#pragma unroll
    for (int k = 0; k < PT_LK; ++k)
        m[k] = (r[k] >= 0 && dst[k] >= 0) ? remap[r[k]] : -1; // r >= 0 always, for a hot sample: pass 1 validated every index
#pragma unroll
    for (int k = 0; k < PT_LK; ++k)
        if (r[k] >= 0 && dst[k] >= 0)
            a.slots[z][dst[k]] = m[k];
}

static int64_t part_tiles(int64_t S) { return (S + PT_TILE - 1) / PT_TILE; }

extern "C" size_t fae_partition_workspace_bytes(const fae_tables *tables, int64_t n_samples)
{
    if (!tables || n_samples < 0)
        return 0;
    size_t S = (size_t)n_samples;
    size_t tiles = (size_t)part_tiles(n_samples);
    return fae_align_up(S * 4 + 4, 256) * 2 + fae_align_up(((size_t)tables->n_tables + 1) * tiles * 4 + 8, 256) + 256;
}

extern "C" int32_t fae_partition_batch(fae_ctx *ctx, const fae_tables *tables, const fae_batch *in,
                                       const int32_t *const *h_remap, int32_t *hot_samples,
                                       int32_t *cold_samples, int64_t *h_n_hot_samples,
                                       int32_t *const *h_slots, int32_t *const *h_hoffsets,
                                       int64_t *h_n_hot_lookups, void *ws, size_t ws_bytes)
{
    int32_t rc = fae_check_tables(ctx, tables, "fae_partition_batch");
    if (rc != FAE_OK)
        return rc;
    rc = fae_check_batch(ctx, tables, in, "fae_partition_batch");
    if (rc != FAE_OK)
        return rc;
    if (!h_remap || !h_n_hot_samples || !h_slots || !h_hoffsets || !h_n_hot_lookups)
        return fae_fail(ctx, FAE_EINVAL, "fae_partition_batch: null argument");
    const int nt = tables->n_tables;
    const int64_t S = in->n_samples;
    if (nt + 2 > FAE_BLK_WORDS - FAE_BLK_SCALARS)
        return fae_fail(ctx, FAE_EINVAL, "fae_partition_batch: too many tables");
    if (S == 0) {
        *h_n_hot_samples = 0;
        for (int z = 0; z < nt; ++z)
            h_n_hot_lookups[z] = 0;
        return FAE_OK;
    }
    if (!hot_samples || !cold_samples)
        return fae_fail(ctx, FAE_EINVAL, "fae_partition_batch: null sample lists");
    if (!ws || ws_bytes < fae_partition_workspace_bytes(tables, S))
        return fae_fail(ctx, FAE_ENOSPC, "fae_partition_batch: workspace too small");
    FAE_HIP(ctx, hipSetDevice(ctx->device));

    PartArgs a;
    memset(&a, 0, sizeof(a));
    const int64_t tiles = part_tiles(S);
    fae_carver cv(ws, ws_bytes);
    a.cold = cv.take<uint32_t>((size_t)S + 1);
    a.hidx = cv.take<int32_t>((size_t)S + 1);
    a.tile_sums = cv.take<int32_t>((size_t)(nt + 1) * tiles + 2);
    if (!cv.ok)
        return fae_fail(ctx, FAE_ENOSPC, "fae_partition_batch: workspace too small");
    int64_t blocks = 0;
    for (int z = 0; z < nt; ++z) {
        if (!h_remap[z] && tables->h_rows[z] > 0)
            return fae_fail(ctx, FAE_EINVAL, "fae_partition_batch: null remap for table %d", z);
        if (!h_hoffsets[z] || (!h_slots[z] && in->h_n_lookups[z] > 0))
            return fae_fail(ctx, FAE_EINVAL, "fae_partition_batch: null outputs for table %d", z);
        a.idx[z] = in->h_indices[z];
        a.wide = in->index_bits == 64;
        a.offsets[z] = in->h_offsets ? in->h_offsets[z] : nullptr;
        a.remap[z] = h_remap[z];
        a.slots[z] = h_slots[z];
        a.hoffsets[z] = h_hoffsets[z];
        a.n_rows[z] = (int32_t)tables->h_rows[z];
        a.n_lookups[z] = (int32_t)in->h_n_lookups[z];
        a.blk_start[z] = (int32_t)blocks;
        blocks += (in->h_n_lookups[z] + PT_BLOCK - 1) / PT_BLOCK;
    }
    a.blk_start[nt] = (int32_t)blocks;
    if (blocks >= 2147483647LL)
        return fae_fail(ctx, FAE_EINVAL, "fae_partition_batch: chunk too large for one launch");
    a.n_tables = nt;
    a.n_samples = (int32_t)S;
    a.n_tiles = (int32_t)tiles;
    a.hot_samples = hot_samples;
    a.cold_samples = cold_samples;
    a.status = ctx->d_block;
    a.scalars = ctx->d_block + FAE_BLK_SCALARS;

    rc = fae_fill_u32(ctx, a.cold, S, 0u);
    if (rc != FAE_OK)
        return rc;
    if (blocks > 0) {
        fae_ktimer kt(ctx, FAE_K_PARTITION);
        FAE_LAUNCH(ctx, part_mark_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, a);
        FAE_LAUNCH_CHECK(ctx);
    }
    {
        fae_ktimer kt(ctx, FAE_K_PARTITION);
        FAE_LAUNCH(ctx, part_count_kernel, dim3((unsigned)tiles, nt + 1), dim3(256), 0, ctx->stream, a);
        FAE_LAUNCH_CHECK(ctx);
    }
    rc = fae_scan_i32(ctx, a.tile_sums, (int64_t)(nt + 1) * tiles);
    if (rc != FAE_OK)
        return rc;
    fae_ktimer kt(ctx, FAE_K_PARTITION);
    FAE_LAUNCH(ctx, part_emit_kernel, dim3((unsigned)tiles), dim3(256), 0, ctx->stream, a);
    FAE_LAUNCH_CHECK(ctx);
    FAE_LAUNCH(ctx, part_offsets_kernel, dim3((unsigned)tiles, nt), dim3(256), 0, ctx->stream, a);
    FAE_LAUNCH_CHECK(ctx);
    if (blocks > 0) {
        FAE_LAUNCH(ctx, part_slots_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, a);
        FAE_LAUNCH_CHECK(ctx);
    }
    rc = fae_readback(ctx, FAE_BLK_SCALARS, nt + 1);
    if (rc != FAE_OK)
        return rc;
    *h_n_hot_samples = (int64_t)ctx->h_block[FAE_BLK_SCALARS];
    for (int z = 0; z < nt; ++z)
        h_n_hot_lookups[z] = (int64_t)ctx->h_block[FAE_BLK_SCALARS + 1 + z];
    return fae_sync_status(ctx);
}
