// Hot mini-batch forward: row gather + sum pooling over HBM-resident hot tables.
//
// One launch covers every table of the batch.  Two lane mappings:
//   group-per-bag : LPR adjacent lanes own one bag, each lane one 16-byte column
//                   slice; bags of a wave sit side by side (best for one-hot / short bags);
//   wave-per-bag  : the 64/LPR lane groups of a wave take alternate entries of one
//                   bag and are combined with cross-lane shuffles (best for long,
//                   uneven bags: no lane group idles while its neighbour finishes).
// Bandwidth bound: per lookup one slot (4 B) and one row (dim*4 B) are read, per bag
// one row is written.  No arithmetic beyond one add per loaded float.
#include "fae_internal.h"
#include "fae_device.h"

struct FwdArgs {
    const float *W[FAE_MAX_TABLES];
    const int32_t *slots[FAE_MAX_TABLES];
    const int32_t *offsets[FAE_MAX_TABLES];
    int32_t n_hot[FAE_MAX_TABLES];
    int32_t n_lookups[FAE_MAX_TABLES];
    int32_t blk_start[FAE_MAX_TABLES + 1];
    int32_t n_tables;
    int32_t dim;
    int32_t n_samples;
    int64_t out_stride;
    float *out;
    uint32_t *status;
    int32_t stream_out; // non-temporal stores for the pooled output
    int32_t mean;       // divide the pooled sum by the bag's length (bags of one lookup are unaffected)
};

// one row slice, or zero (and a status flag) when the slot is out of range
template <typename V>
__device__ __forceinline__ V fwd_load(const V *W, int slot, int n_hot, int ncols, int c, uint32_t *status)
{
    if ((unsigned)slot >= (unsigned)n_hot) {
        fae_flag(status, FAE_STATUS_ERANGE);
        return vec_ops<V>::zero();
    }
    return W[(int64_t)slot * ncols + c];
}

// Sum of the rows of lookups j0, j0 + step, ... below end (column slice c), four loads in flight.
// Up to FWD_PLAIN_MAX terms are added one after the other (worst case FWD_PLAIN_MAX * 2^-24 of
// the sum of their magnitudes, inside the 1e-5 the result is held to); longer sums carry the
// rounding error along (COMP), so that a bag of thousands of lookups stays as accurate as a short
// one, also when it adds one popular row over and over, which otherwise drifts one way.
#define FWD_PLAIN_MAX 128
template <typename V, bool COMP>
__device__ __forceinline__ V fwd_sum(const V *W, const int32_t *slots, int j0, int end, int step, int n_hot, int ncols, int c,
                                     uint32_t *status)
{
    V acc = vec_ops<V>::zero(), lost = vec_ops<V>::zero();
    int j = j0;
    for (; j + 3 * step < end; j += 4 * step) {
        const int s0 = slots[j], s1 = slots[j + step], s2 = slots[j + 2 * step], s3 = slots[j + 3 * step];
        const V v0 = fwd_load(W, s0, n_hot, ncols, c, status);
        const V v1 = fwd_load(W, s1, n_hot, ncols, c, status);
        const V v2 = fwd_load(W, s2, n_hot, ncols, c, status);
        const V v3 = fwd_load(W, s3, n_hot, ncols, c, status);
        if (COMP) {
            vec_ops<V>::add_comp(acc, lost, v0);
            vec_ops<V>::add_comp(acc, lost, v1);
            vec_ops<V>::add_comp(acc, lost, v2);
            vec_ops<V>::add_comp(acc, lost, v3);
        } else {
            vec_ops<V>::add(acc, v0);
            vec_ops<V>::add(acc, v1);
            vec_ops<V>::add(acc, v2);
            vec_ops<V>::add(acc, v3);
        }
    }
    for (; j < end; j += step) {
        const V v = fwd_load(W, slots[j], n_hot, ncols, c, status);
        if (COMP)
            vec_ops<V>::add_comp(acc, lost, v);
        else
            vec_ops<V>::add(acc, v);
    }
    return acc;
}

template <typename V, int LPR> __global__ __launch_bounds__(256) void fwd_group_kernel(FwdArgs a)
{
    constexpr int GPB = 256 / LPR;
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int bl = blockIdx.x - a.blk_start[z];
    const int g = threadIdx.x / LPR, l = threadIdx.x % LPR;
    const int64_t s = (int64_t)bl * GPB + g;
    if (s >= a.n_samples)
        return;
    const int32_t *off = a.offsets[z];
    const int32_t *slots = a.slots[z];
    int beg = off ? off[s] : (int)s;
    int end = off ? off[s + 1] : (int)s + 1;
    if (beg < 0 || end > a.n_lookups[z] || beg > end) { // malformed CSR: never dereferenced
        fae_flag(a.status, FAE_STATUS_ERANGE);
        end = beg = 0;
    }
    const int ncols = a.dim / (int)(sizeof(V) / sizeof(float));
    const V *W = (const V *)a.W[z];
    const int n_hot = a.n_hot[z];
    V *o = (V *)(a.out + s * a.out_stride + (int64_t)z * a.dim);
    for (int c = l; c < ncols; c += LPR) {
        const V acc = end - beg > FWD_PLAIN_MAX ? fwd_sum<V, true>(W, slots, beg, end, 1, n_hot, ncols, c, a.status)
                                                : fwd_sum<V, false>(W, slots, beg, end, 1, n_hot, ncols, c, a.status);
        V res = acc;
        if (a.mean && end - beg > 1)
            vec_ops<V>::scale(res, 1.0f / (float)(end - beg));
        o[c] = res;
    }
}

// One-hot tables: 256 samples per workgroup, 64 per wave.
template <typename V, int LPR> __global__ __launch_bounds__(256) void fwd_onehot_kernel(FwdArgs a)
{
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int bl = blockIdx.x - a.blk_start[z];
    const int64_t s0 = ((int64_t)bl * (256 / FAE_WAVE) + threadIdx.x / FAE_WAVE) * FAE_WAVE;
    fwd_onehot_wave<V, LPR>((const V *)a.W[z], a.slots[z], a.n_hot[z], s0, a.n_samples, a.out + (int64_t)z * a.dim,
                            a.out_stride, a.dim, a.status, a.stream_out != 0);
}

template <typename V, int LPR> __global__ __launch_bounds__(256) void fwd_wave_kernel(FwdArgs a)
{
    constexpr int G = FAE_WAVE / LPR; // lane groups per wave
    constexpr int WPB = 256 / FAE_WAVE;
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int bl = blockIdx.x - a.blk_start[z];
    const int w = threadIdx.x / FAE_WAVE, lane = threadIdx.x % FAE_WAVE;
    const int g = lane / LPR, l = lane % LPR;
    const int64_t s = (int64_t)bl * WPB + w;
    if (s >= a.n_samples)
        return;
    const int32_t *off = a.offsets[z];
    const int32_t *slots = a.slots[z];
    int beg = off ? off[s] : (int)s;
    int end = off ? off[s + 1] : (int)s + 1;
    if (beg < 0 || end > a.n_lookups[z] || beg > end) { // malformed CSR: never dereferenced
        fae_flag(a.status, FAE_STATUS_ERANGE);
        end = beg = 0;
    }
    const int ncols = a.dim / (int)(sizeof(V) / sizeof(float));
    const V *W = (const V *)a.W[z];
    const int n_hot = a.n_hot[z];
    V *o = (V *)(a.out + s * a.out_stride + (int64_t)z * a.dim);
    for (int c0 = 0; c0 < ncols; c0 += LPR) {
        const int c = c0 + l;
        V acc = vec_ops<V>::zero();
        if (c < ncols) // every group sums every G-th lookup of the bag (the bag's length is the same for the whole wave)
            acc = end - beg > FWD_PLAIN_MAX * G ? fwd_sum<V, true>(W, slots, beg + g, end, G, n_hot, ncols, c, a.status)
                                                : fwd_sum<V, false>(W, slots, beg + g, end, G, n_hot, ncols, c, a.status);
        // combine the lane groups (all 64 lanes take part in the shuffles)
#pragma unroll
        for (int m = LPR; m < FAE_WAVE; m <<= 1)
            vec_ops<V>::add(acc, vec_ops<V>::shfl_xor(acc, m));
        if (a.mean && end - beg > 1)
            vec_ops<V>::scale(acc, 1.0f / (float)(end - beg));
        if (g == 0 && c < ncols)
            o[c] = acc;
    }
}

template <typename V, int LPR> static void fwd_launch(fae_ctx *ctx, const FwdArgs &a, int kind, int total_blocks)
{
    if (kind == 2)
        FAE_LAUNCH(ctx, (fwd_onehot_kernel<V, LPR>), dim3(total_blocks), dim3(256), 0, ctx->stream, a);
    else if (kind == 1)
        FAE_LAUNCH(ctx, (fwd_wave_kernel<V, LPR>), dim3(total_blocks), dim3(256), 0, ctx->stream, a);
    else
        FAE_LAUNCH(ctx, (fwd_group_kernel<V, LPR>), dim3(total_blocks), dim3(256), 0, ctx->stream, a);
}

template <typename V> static void fwd_dispatch(fae_ctx *ctx, const FwdArgs &a, int lpr, int kind, int total_blocks)
{
    switch (lpr) {
    case 1: fwd_launch<V, 1>(ctx, a, kind, total_blocks); break;
    case 2: fwd_launch<V, 2>(ctx, a, kind, total_blocks); break;
    case 4: fwd_launch<V, 4>(ctx, a, kind, total_blocks); break;
    case 8: fwd_launch<V, 8>(ctx, a, kind, total_blocks); break;
    case 16: fwd_launch<V, 16>(ctx, a, kind, total_blocks); break;
    case 32: fwd_launch<V, 32>(ctx, a, kind, total_blocks); break;
    default: fwd_launch<V, 64>(ctx, a, kind, total_blocks); break;
    }
}

static int32_t fwd_impl(fae_ctx *ctx, const fae_tables *hot_tables, const float *const *h_hotW,
                        const fae_batch *hot_batch, float *out, int64_t out_row_stride, int pooling);

extern "C" int32_t fae_embbag_fwd(fae_ctx *ctx, const fae_tables *hot_tables, const float *const *h_hotW,
                                  const fae_batch *hot_batch, float *out, int64_t out_row_stride)
{
    return fwd_impl(ctx, hot_tables, h_hotW, hot_batch, out, out_row_stride, FAE_POOL_SUM);
}

extern "C" int32_t fae_embbag_fwd_opts(fae_ctx *ctx, const fae_tables *hot_tables, const float *const *h_hotW,
                                       const fae_batch *hot_batch, float *out, int64_t out_row_stride,
                                       const fae_step_opts *opts)
{
    if (!ctx)
        return FAE_EINVAL;
    if (!opts || (opts->pooling != FAE_POOL_SUM && opts->pooling != FAE_POOL_MEAN))
        return fae_fail(ctx, FAE_EINVAL, "fae_embbag_fwd_opts: null options or unknown pooling");
    return fwd_impl(ctx, hot_tables, h_hotW, hot_batch, out, out_row_stride, opts->pooling);
}

static int32_t fwd_impl(fae_ctx *ctx, const fae_tables *hot_tables, const float *const *h_hotW,
                        const fae_batch *hot_batch, float *out, int64_t out_row_stride, int pooling)
{
    int32_t rc = fae_check_tables(ctx, hot_tables, "fae_embbag_fwd");
    if (rc != FAE_OK)
        return rc;
    rc = fae_check_batch(ctx, hot_tables, hot_batch, "fae_embbag_fwd");
    if (rc != FAE_OK)
        return rc;
    if (hot_batch->index_bits == 64)
        return fae_fail(ctx, FAE_EINVAL, "fae_embbag_fwd: hot slots are int32");
    const int nt = hot_tables->n_tables, dim = hot_tables->dim;
    const int64_t S = hot_batch->n_samples;
    if (S == 0)
        return FAE_OK;
    if (!h_hotW || !out || out_row_stride < (int64_t)nt * dim)
        return fae_fail(ctx, FAE_EINVAL, "fae_embbag_fwd: null output/weights or out_row_stride < n_tables*dim");
    FAE_HIP(ctx, hipSetDevice(ctx->device));

    FwdArgs a;
    memset(&a, 0, sizeof(a));
    bool vec = (dim % 4 == 0) && (out_row_stride % 4 == 0) && (((uintptr_t)out) % 16 == 0);
    for (int z = 0; z < nt; ++z) {
        if (!h_hotW[z] && hot_tables->h_rows[z] > 0)
            return fae_fail(ctx, FAE_EINVAL, "fae_embbag_fwd: null weights for table %d", z);
        a.W[z] = h_hotW[z];
        a.slots[z] = hot_batch->h_indices[z];
        a.offsets[z] = hot_batch->h_offsets ? hot_batch->h_offsets[z] : nullptr;
        a.n_hot[z] = (int32_t)hot_tables->h_rows[z];
        a.n_lookups[z] = (int32_t)hot_batch->h_n_lookups[z];
        if (((uintptr_t)h_hotW[z]) % 16 != 0)
            vec = false;
    }
    const int ncols = vec ? dim / 4 : dim;
    int lpr = 1;
    while (lpr < ncols && lpr < 64)
        lpr <<= 1;
    const int groups = 64 / lpr;
    a.n_tables = nt;
    a.dim = dim;
    a.n_samples = (int32_t)S;
    a.out_stride = out_row_stride;
    a.out = out;
    a.status = ctx->d_block;
    a.stream_out = ctx->opt_fwd_stream != 0;
    a.mean = pooling == FAE_POOL_MEAN;
    // one-hot tables: 256 samples per workgroup
    if (ctx->opt_fwd == 0) {
        const int64_t per_table = (S + 255) / 256;
        int64_t blocks = 0;
        for (int z = 0; z < nt; ++z) {
            a.blk_start[z] = (int32_t)blocks;
            if (!a.offsets[z])
                blocks += per_table;
        }
        a.blk_start[nt] = (int32_t)blocks;
        if (blocks >= 2147483647LL)
            return fae_fail(ctx, FAE_EINVAL, "fae_embbag_fwd: batch too large for one launch");
        if (blocks > 0) {
            fae_ktimer kt(ctx, FAE_K_FWD);
            if (vec)
                fwd_dispatch<float4>(ctx, a, lpr, 2, (int)blocks);
            else
                fwd_dispatch<float>(ctx, a, lpr, 2, (int)blocks);
            FAE_LAUNCH_CHECK(ctx);
        }
    }
    // tables with offsets (and every table when a lane mapping is forced)
    {
        int64_t csr_lookups = 0;
        int n_csr = 0;
        for (int z = 0; z < nt; ++z)
            if (a.offsets[z] || ctx->opt_fwd != 0) {
                csr_lookups += hot_batch->h_n_lookups[z];
                ++n_csr;
            }
        if (n_csr > 0) {
            // wave-per-bag pays once a bag keeps every lane group of the wave busy for a few rounds
            const double avg_len = (double)csr_lookups / ((double)S * n_csr);
            bool wave = groups > 1 && avg_len >= 2.0 * groups;
            if (ctx->opt_fwd == 1)
                wave = false;
            if (ctx->opt_fwd == 2)
                wave = groups > 1;
            const int bags_per_block = wave ? 4 : 256 / lpr;
            const int64_t per_table = (S + bags_per_block - 1) / bags_per_block;
            int64_t blocks = 0;
            for (int z = 0; z < nt; ++z) {
                a.blk_start[z] = (int32_t)blocks;
                if (a.offsets[z] || ctx->opt_fwd != 0)
                    blocks += per_table;
            }
            a.blk_start[nt] = (int32_t)blocks;
            if (blocks >= 2147483647LL)
                return fae_fail(ctx, FAE_EINVAL, "fae_embbag_fwd: batch too large for one launch");
            fae_ktimer kt(ctx, FAE_K_FWD);
            if (vec)
                fwd_dispatch<float4>(ctx, a, lpr, wave ? 1 : 0, (int)blocks);
            else
                fwd_dispatch<float>(ctx, a, lpr, wave ? 1 : 0, (int)blocks);
            FAE_LAUNCH_CHECK(ctx);
        }
    }
    return FAE_OK;
}
