// Embedding synchronisation between the hot tables and the full tables (Sec. 3 (4);
// Sec. 6.2, "Embedding Synchronization"): when training switches between hot and cold
// mini-batches, the hot rows are copied back to their places in the full tables, or
// fetched from there again.  One launch covers all tables.
//
// A pure row copy: per hot row 4 bytes of id, dim*4 bytes read and dim*4 bytes written.
// The hot side is a stream; the full-table side is rows of dim*4 bytes at ascending but
// scattered addresses (hot ids ascend with the slot).  A lane moves 16 bytes, a thread
// has four independent copies in flight.
#include "fae_internal.h"

#define SYNC_THREADS 256
#define SYNC_UNROLL 4

struct SyncArgs {
    float *hotW[FAE_MAX_TABLES];
    float *W[FAE_MAX_TABLES];
    const int32_t *hot_ids[FAE_MAX_TABLES];
    int64_t rows[FAE_MAX_TABLES];
    int64_t n_vec[FAE_MAX_TABLES];         // n_hot_z * (dim / vector width)
    int64_t blk_start[FAE_MAX_TABLES + 1]; // 64-bit: a 64 GiB hot set has more than 2^31 vectors
    int32_t n_tables, dim, to_full;
    uint32_t *status;
};

template <typename V> __global__ __launch_bounds__(SYNC_THREADS) void sync_rows_kernel(SyncArgs a)
{
    constexpr int VW = sizeof(V) / sizeof(float);
    int z = 0;
    const int64_t b = blockIdx.x;
    while (z + 1 < a.n_tables && b >= a.blk_start[z + 1])
        ++z;
    const int ncols = a.dim / VW;
    const int64_t e0 = (b - a.blk_start[z]) * (SYNC_THREADS * SYNC_UNROLL) + threadIdx.x;
    const int32_t *ids = a.hot_ids[z];
    V *hot = (V *)a.hotW[z];
    V *full = (V *)a.W[z];
    int64_t src[SYNC_UNROLL], dst[SYNC_UNROLL];
    bool bad = false;
#pragma unroll
    for (int k = 0; k < SYNC_UNROLL; ++k) {
        const int64_t e = e0 + (int64_t)k * SYNC_THREADS;
        src[k] = dst[k] = -1;
        if (e < a.n_vec[z]) {
            const int64_t slot = e / ncols;
            const int c = (int)(e - slot * ncols);
            const int64_t row = ids[slot];
            if (row < 0 || row >= a.rows[z]) {
                bad = true; // never dereferenced
            } else {
                const int64_t f = row * ncols + c;
                src[k] = a.to_full ? e : f;
                dst[k] = a.to_full ? f : e;
            }
        }
    }
    const V *from = a.to_full ? hot : full;
    V *to = a.to_full ? full : hot;
    V v[SYNC_UNROLL];
#pragma unroll
    for (int k = 0; k < SYNC_UNROLL; ++k)
        if (src[k] >= 0)
            v[k] = from[src[k]];
#pragma unroll
    for (int k = 0; k < SYNC_UNROLL; ++k)
        if (src[k] >= 0)
            to[dst[k]] = v[k];
    if (bad)
        fae_flag(a.status, FAE_STATUS_ERANGE);
}

extern "C" int32_t fae_sync_hot_rows(fae_ctx *ctx, const fae_tables *tables, const int64_t *h_n_hot,
                                     const int32_t *const *h_hot_ids, float *const *h_hotW,
                                     float *const *h_W, int32_t direction)
{
    int32_t rc = fae_check_tables(ctx, tables, "fae_sync_hot_rows");
    if (rc != FAE_OK)
        return rc;
    if (!h_n_hot || !h_hot_ids || !h_hotW || !h_W)
        return fae_fail(ctx, FAE_EINVAL, "fae_sync_hot_rows: null argument");
    if (direction != FAE_SYNC_HOT_TO_FULL && direction != FAE_SYNC_FULL_TO_HOT)
        return fae_fail(ctx, FAE_EINVAL, "fae_sync_hot_rows: unknown direction %d", direction);
    const int nt = tables->n_tables, dim = tables->dim;
    bool vec = dim % 4 == 0;
    SyncArgs a;
    memset(&a, 0, sizeof(a));
    for (int z = 0; z < nt; ++z) {
        if (h_n_hot[z] < 0 || h_n_hot[z] > tables->h_rows[z])
            return fae_fail(ctx, FAE_EINVAL, "fae_sync_hot_rows: n_hot[%d]=%lld outside [0, rows]", z,
                            (long long)h_n_hot[z]);
        if (h_n_hot[z] > 0 && (!h_hot_ids[z] || !h_hotW[z] || !h_W[z]))
            return fae_fail(ctx, FAE_EINVAL, "fae_sync_hot_rows: null pointer for table %d", z);
        vec = vec && ((((uintptr_t)h_hotW[z]) | ((uintptr_t)h_W[z])) & 15) == 0;
    }
    const int vw = vec ? 4 : 1;
    int64_t blocks = 0;
    for (int z = 0; z < nt; ++z) {
        a.hotW[z] = h_hotW[z];
        a.W[z] = h_W[z];
        a.hot_ids[z] = h_hot_ids[z];
        a.rows[z] = tables->h_rows[z];
        a.n_vec[z] = h_n_hot[z] * (dim / vw);
        a.blk_start[z] = blocks;
        blocks += (a.n_vec[z] + SYNC_THREADS * SYNC_UNROLL - 1) / (SYNC_THREADS * SYNC_UNROLL);
    }
    a.blk_start[nt] = blocks;
    a.n_tables = nt;
    a.dim = dim;
    a.to_full = direction == FAE_SYNC_HOT_TO_FULL;
    a.status = ctx->d_block;
    if (blocks == 0)
        return FAE_OK;
    if (blocks > 2147483647LL)
        return fae_fail(ctx, FAE_EINVAL, "fae_sync_hot_rows: more than 2^31 workgroups; split the call by tables");
    FAE_HIP(ctx, hipSetDevice(ctx->device));
    fae_ktimer kt(ctx, FAE_K_SYNC_ROWS);
    if (vec)
        FAE_LAUNCH(ctx, sync_rows_kernel<float4>, dim3((unsigned)blocks), dim3(SYNC_THREADS), 0, ctx->stream, a);
    else
        FAE_LAUNCH(ctx, sync_rows_kernel<float>, dim3((unsigned)blocks), dim3(SYNC_THREADS), 0, ctx->stream, a);
    FAE_LAUNCH_CHECK(ctx);
    return FAE_OK;
}
