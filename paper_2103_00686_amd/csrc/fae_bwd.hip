// Hot mini-batch backward + sparse SGD (Sec. 2.2 "optimizer on embeddings", Sec. 6.2:
// embedding update on the GPU for hot mini-batches).
//
//   1. keys    key = hot slot, value = sample id, per table segment
//   2. sort    stable sort of (key, value), segmented by table: inside LDS for tables of up
//              to 16 K lookups, else LSD radix passes over only the bits a hot slot can
//              occupy (one chained kernel per pass for short lists, three kernels per pass
//              for long ones)
//   3. reduce  one wave owns a span of the sorted lookups.  Its 64/LPR lane groups
//              take consecutive lookups (LPR lanes x 16 B cover one gradient row); a
//              segmented scan over the groups, which also hands on the sum carried
//              from the previous step, sums each run of equal keys; a run that lies
//              inside the span gets its update w -= lr * G at once.  All gradient loads
//              of a span are independent of the run structure, so they pipeline freely.
//   4. borders the first / last run of a span may continue in the neighbours: those
//              sums are published in a small scratch array and the span in which the
//              run ends adds them in span order and applies the update (inside the
//              reduce kernel; as a kernel of its own for very wide rows or on request).
// No float atomics: every row has exactly one writer, and the summation order is fixed by the
// stable sort (the optional counting sort, sort_order=1, leaves the order inside a run open).
// Bandwidth bound: per lookup one gradient row is read, per distinct row one weight
// row is read and written; the sort moves 16 B per lookup and pass.
//
// This file: workspace layout, argument set-up and the entry points.  Steps 1 + 2 are in
// fae_bwd_sort.hip, steps 3 + 4 in fae_bwd_reduce.hip, what they share in fae_bwd.h.
#include "fae_bwd.h"

#include <mutex>

// ---------------------------------------------------------------------------------
// plan and workspace
// ---------------------------------------------------------------------------------
BwdPlan bwd_plan(int nt, const int64_t *h_n_lookups)
{
    BwdPlan p;
    p.N = 0;
    p.tiles = 0;
    p.small_tiles = 0;
    p.max_spans = 0;
    for (int z = 0; z < nt; ++z) {
        p.N += h_n_lookups[z];
        p.tiles += (h_n_lookups[z] + SORT_TILE - 1) / SORT_TILE;
        p.small_tiles += (h_n_lookups[z] + SORT_TILE_SMALL - 1) / SORT_TILE_SMALL;
        p.max_spans += (h_n_lookups[z] + BWD_SPAN_MIN - 1) / BWD_SPAN_MIN;
    }
    p.dbg_tiles = (p.N + DBG_TILE - 1) / DBG_TILE;
    return p;
}

// lookups per wave: long spans amortise the border handling, short ones fill the chip
int bwd_span(const BwdPlan &p, int n_cu)
{
    int span = BWD_SPAN_MAX;
    while (span > BWD_SPAN_MIN && p.N / span < 8LL * n_cu)
        span >>= 1;
    return span;
}


BwdWs bwd_carve(void *ws, size_t bytes, const BwdPlan &p, int nt, int dim, int span)
{
    fae_carver cv(ws, bytes);
    BwdWs w;
    for (int i = 0; i < 2; ++i) {
        w.keys[i] = cv.take<int32_t>((size_t)p.N + 1);
        w.vals[i] = cv.take<int32_t>((size_t)p.N + 1);
    }
    w.hist = cv.take<int32_t>((size_t)RADIX * p.tiles + 1);
    w.tot = cv.take<int32_t>((size_t)nt * RADIX);
    const size_t sweep_tiles = p.small_tiles <= SORT_SMALL_MAX_TILES ? (size_t)p.small_tiles : (size_t)p.tiles;
    w.n_flags = p.max_spans + nt + 1;
    w.flags = cv.take<int32_t>((size_t)w.n_flags); // directly in front of the sweep area: one fill clears both
    w.sweep = cv.take<uint32_t>(64 + ((size_t)nt + sweep_tiles) * SWEEP_MAX_PASSES * RADIX);
    w.partial = cv.take<float>((size_t)(p.max_spans * BWD_SPAN_MIN / span + nt + 1) * 2 * dim);
    w.dbg_tile_sums = cv.take<int32_t>((size_t)p.dbg_tiles + 2);
    w.dbg_rstart = cv.take<int32_t>((size_t)p.N + 2);
    w.ok = cv.ok;
    w.used = cv.used;
    return w;
}

extern "C" size_t fae_bwd_workspace_bytes(const fae_tables *hot_tables, int64_t n_samples, const int64_t *h_n_lookups)
{
    (void)n_samples;
    if (!hot_tables || !h_n_lookups || hot_tables->n_tables < 1 || hot_tables->n_tables > FAE_MAX_TABLES)
        return 0;
    BwdPlan p = bwd_plan(hot_tables->n_tables, h_n_lookups);
    // sized for the smallest span, so the size does not depend on the device's CU count
    BwdWs w = bwd_carve((void *)256, (size_t)-1, p, hot_tables->n_tables, hot_tables->dim, BWD_SPAN_MIN);
    return w.used + 256;
}

int32_t bwd_setup(fae_ctx *ctx, const fae_tables *hot_tables, const fae_batch *hot_batch, void *ws, size_t ws_bytes,
                  const char *who, BwdSetup *out)
{
    int32_t rc = fae_check_tables(ctx, hot_tables, who);
    if (rc != FAE_OK)
        return rc;
    rc = fae_check_batch(ctx, hot_tables, hot_batch, who);
    if (rc != FAE_OK)
        return rc;
    if (hot_batch->index_bits == 64)
        return fae_fail(ctx, FAE_EINVAL, "%s: hot slots are int32", who);
    const int nt = hot_tables->n_tables, dim = hot_tables->dim;
    out->plan = bwd_plan(nt, hot_batch->h_n_lookups);
    if (out->plan.N >= 2147483647LL - SORT_TILE)
        return fae_fail(ctx, FAE_EINVAL, "%s: more than 2^31 lookups in one call", who);
    out->empty = out->plan.N == 0 || hot_batch->n_samples == 0;
    if (out->empty)
        return FAE_OK;
    if (!ws)
        return fae_fail(ctx, FAE_ENOSPC, "%s: null workspace", who);
    out->w = bwd_carve(ws, ws_bytes, out->plan, nt, dim, BWD_SPAN_MIN);
    if (!out->w.ok)
        return fae_fail(ctx, FAE_ENOSPC, "%s: workspace too small (%zu needed)", who, out->w.used);
    BwdArgs &a = out->a;
    memset(&a, 0, sizeof(a));
    int64_t lookups = 0;
    for (int z = 0; z < nt; ++z) {
        a.slots[z] = hot_batch->h_indices[z];
        a.offsets[z] = hot_batch->h_offsets ? hot_batch->h_offsets[z] : nullptr;
        a.n_hot[z] = (int32_t)hot_tables->h_rows[z];
        a.seg_start[z] = (int32_t)lookups;
        lookups += hot_batch->h_n_lookups[z];
    }
    a.seg_start[nt] = (int32_t)lookups;
    a.n_tables = nt;
    a.dim = dim;
    a.n_samples = (int32_t)hot_batch->n_samples;
    a.hist = out->w.hist;
    a.tot = out->w.tot;
    a.partial = out->w.partial;
    a.flags = out->w.flags;
    a.n_flags = (int32_t)out->w.n_flags;
    a.status = ctx->d_block;
    return FAE_OK;
}

static int32_t bwd_impl(fae_ctx *ctx, const fae_tables *hot_tables, float *const *h_hotW,
                        const fae_batch *hot_batch, const float *gout, int64_t gout_row_stride,
                        const fae_step_opts &opts, const fae_bwd_debug *dbg, void *ws, size_t ws_bytes);

extern "C" int32_t fae_embbag_bwd_sgd(fae_ctx *ctx, const fae_tables *hot_tables, float *const *h_hotW,
                                      const fae_batch *hot_batch, const float *gout, int64_t gout_row_stride,
                                      float lr, const fae_bwd_debug *dbg, void *ws, size_t ws_bytes)
{
    fae_step_opts o;
    memset(&o, 0, sizeof(o));
    o.pooling = FAE_POOL_SUM;
    o.optimizer = FAE_OPT_SGD;
    o.lr = lr;
    return bwd_impl(ctx, hot_tables, h_hotW, hot_batch, gout, gout_row_stride, o, dbg, ws, ws_bytes);
}

extern "C" int32_t fae_embbag_bwd_opts(fae_ctx *ctx, const fae_tables *hot_tables, float *const *h_hotW,
                                       const fae_batch *hot_batch, const float *gout, int64_t gout_row_stride,
                                       const fae_step_opts *opts, const fae_bwd_debug *dbg, void *ws,
                                       size_t ws_bytes)
{
    if (!ctx)
        return FAE_EINVAL;
    if (!opts || (opts->pooling != FAE_POOL_SUM && opts->pooling != FAE_POOL_MEAN) ||
        (opts->optimizer != FAE_OPT_SGD && opts->optimizer != FAE_OPT_ROWWISE_ADAGRAD))
        return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_opts: null options, unknown pooling or unknown optimizer");
    if (opts->optimizer == FAE_OPT_ROWWISE_ADAGRAD) {
        if (!opts->h_state || !(opts->eps >= 0.f))
            return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_opts: Adagrad needs accumulators and eps >= 0");
        if (hot_tables && (hot_tables->dim > 256 || (hot_tables->dim % 4 != 0 && hot_tables->dim > 64)))
            return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_opts: Adagrad needs dim <= 256 (<= 64 if dim %% 4 != 0)");
    }
    return bwd_impl(ctx, hot_tables, h_hotW, hot_batch, gout, gout_row_stride, *opts, dbg, ws, ws_bytes);
}

// The second form of the reduce kernel addresses rows with 24-bit by 24-bit multiplies and 32-bit byte offsets
// and handles float4 columns that fit one pass over a lane group of 4 to 64 lanes: true where all of
// that holds.
static bool bwd_walk_fits(const fae_tables *hot_tables, const fae_batch *hot_batch, int64_t gout_row_stride,
                          bool vec, int ncols, int lpr)
{
    const int64_t lim24 = (int64_t)1 << 24, lim32 = (int64_t)1 << 32;
    const int64_t rowb = (int64_t)hot_tables->dim * 4, gstrideb = gout_row_stride * 4;
    if (!vec || ncols > lpr || lpr < 4 || rowb >= lim24 || gstrideb >= lim24 || hot_batch->n_samples > lim24 ||
        hot_batch->n_samples * gstrideb >= lim32)
        return false;
    for (int z = 0; z < hot_tables->n_tables; ++z)
        if (hot_tables->h_rows[z] > lim24 || hot_tables->h_rows[z] * rowb >= lim32)
            return false;
    return true;
}

static int32_t bwd_impl(fae_ctx *ctx, const fae_tables *hot_tables, float *const *h_hotW,
                        const fae_batch *hot_batch, const float *gout, int64_t gout_row_stride,
                        const fae_step_opts &opts, const fae_bwd_debug *dbg, void *ws, size_t ws_bytes)
{
    const float lr = opts.lr;
    if (dbg && !dbg->table_start)
        return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_sgd: incomplete debug outputs");
    BwdSetup su;
    int32_t rc = bwd_setup(ctx, hot_tables, hot_batch, ws, ws_bytes, "fae_embbag_bwd_sgd", &su);
    if (rc != FAE_OK)
        return rc;
    const int nt = hot_tables->n_tables, dim = hot_tables->dim;
    FAE_HIP(ctx, hipSetDevice(ctx->device));
    if (su.empty) { // nothing to update
        if (dbg) {
            rc = fae_fill_u32(ctx, dbg->table_start, nt + 1, 0u);
            if (rc != FAE_OK)
                return rc;
        }
        return FAE_OK;
    }
    if (!h_hotW || !gout || gout_row_stride < (int64_t)nt * dim)
        return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_sgd: null gradient/weights or gout_row_stride < n_tables*dim");
    if (dbg && (!dbg->uniq || !dbg->runlen))
        return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_sgd: incomplete debug outputs");
    const BwdPlan &plan = su.plan;
    const BwdWs &w = su.w;
    BwdArgs &a = su.a;
    const int span = ctx->opt_span ? (int)ctx->opt_span : bwd_span(plan, ctx->n_cu);
    bool vec = (dim % 4 == 0) && (gout_row_stride % 4 == 0) && (((uintptr_t)gout) % 16 == 0);
    for (int z = 0; z < nt; ++z) {
        if (!h_hotW[z] && hot_tables->h_rows[z] > 0)
            return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_sgd: null weights for table %d", z);
        a.W[z] = h_hotW[z];
        if (((uintptr_t)h_hotW[z]) % 16 != 0)
            vec = false;
    }
    a.gout = gout;
    a.gout_stride = gout_row_stride;
    a.lr = lr;
    a.span = span;
    a.mean = opts.pooling == FAE_POOL_MEAN;
    a.adagrad = opts.optimizer == FAE_OPT_ROWWISE_ADAGRAD;
    a.eps = opts.eps;
    if (a.adagrad) {
        for (int z = 0; z < nt; ++z) {
            if (!opts.h_state[z] && hot_tables->h_rows[z] > 0)
                return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_opts: null accumulators for table %d", z);
            a.opt_state[z] = opts.h_state[z];
        }
        if (!vec && dim > 64) // the unaligned path has one column per lane
            return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_opts: Adagrad on unaligned buffers needs dim <= 64");
    }

    // 1 + 2. sorted (slot, sample) pairs: take them from a matching presort, or sort now
    int cur = 0;
    fae_ctx::Presort *ps = ctx->presort_find(ws);
    if (ps && ps->side) {
        // whatever the side stream was asked to do in this workspace must be finished before it is used
        FAE_HIP(ctx, hipStreamWaitEvent(ctx->stream, ps->ev_join, 0));
    }
    if (ps && fae_ctx::presort_is(ps, nt, hot_batch)) {
        cur = ps->cur;
    } else {
        rc = bwd_sort_stage(ctx, ctx->stream, hot_tables, hot_batch, su, &cur);
        if (rc != FAE_OK)
            return rc;
    }
    if (ps)
        ps->valid = false;
    a.keys_in = w.keys[cur];
    a.vals_in = w.vals[cur];
    a.keys_out = nullptr;
    a.vals_out = nullptr;

    // 3 + 4. reduce + SGD, then the runs that cross span borders
    const int ncols = vec ? dim / 4 : dim;
    int lpr = 1;
    while (lpr < ncols && lpr < 64)
        lpr <<= 1;
    {
        int64_t spans = 0;
        for (int z = 0; z < nt; ++z) {
            a.blk_start[z] = (int32_t)spans;
            spans += (hot_batch->h_n_lookups[z] + span - 1) / span;
        }
        a.blk_start[nt] = (int32_t)spans;
        a.n_spans = (int32_t)spans;
        // runs that cross span borders: finished inside the reduce kernel (scan form, rows that fit
        // one pass over the lanes), else by the fix-up kernel
        a.form = 0;
        // one wave per workgroup unless asked otherwise: the waves of a launch then spread evenly
        // over the compute units whatever the number of spans is
        a.wg_waves = ctx->opt_wg_waves ? (int32_t)ctx->opt_wg_waves : 1;
        if (ctx->opt_reduce == 2 && !a.mean && !a.adagrad &&
            bwd_walk_fits(hot_tables, hot_batch, gout_row_stride, vec, ncols, lpr))
            a.form = 1;
        a.fused_fixup = ctx->opt_fixup != 1 && ncols <= lpr && spans <= a.n_flags;
        a.handoff = ctx->opt_handoff == 1 ? 1 : 0;
        bwd_launch_reduce(ctx, a, vec, lpr);
        FAE_LAUNCH_CHECK(ctx);
    }
    // optional: distinct slots and multiplicities
    if (dbg) {
        a.dbg_uniq = dbg->uniq;
        a.dbg_runlen = dbg->runlen;
        a.dbg_table_start = dbg->table_start;
        a.dbg_tile_sums = w.dbg_tile_sums;
        a.dbg_rstart = w.dbg_rstart;
        a.dbg_tiles = (int32_t)plan.dbg_tiles;
        rc = bwd_launch_debug(ctx, a);
        if (rc != FAE_OK)
            return rc;
    }
    return FAE_OK;
}

// ---------------------------------------------------------------------------------
// The backward for callers that cannot allocate: the workspace lives inside the library.
// ---------------------------------------------------------------------------------
// One array per device (every device that loads the library's code object holds its own copy at
// its own address until the process ends).  In host code the array's name only stands for the
// symbol: the device address comes from hipGetSymbolAddress, once per device with that device
// current, and is what every launch and fill is given.
static __device__ __align__(256) unsigned char fae_bwd_scratch[FAE_BWD_STATIC_WS_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {nullptr};
} // namespace

// Device address of this device's copy of the array (resolved at most once per device).  The
// caller has made `device` current.
int32_t fae_bwd_scratch_resolve(fae_ctx *ctx, int device, void **out)
{
    *out = nullptr;
    if (device < 0 || device >= kMaxDevices)
        return fae_fail(ctx, FAE_EINVAL, "built-in workspace: device %d outside [0,%d)", device, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        FAE_HIP(ctx, hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(fae_bwd_scratch)));
        if (!ptr)
            return fae_fail(ctx, FAE_EHIP, "built-in workspace: no device address for device %d", device);
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return FAE_OK;
}

extern "C" size_t fae_bwd_static_workspace_bytes(void) { return (size_t)FAE_BWD_STATIC_WS_BYTES; }

extern "C" int32_t fae_embbag_bwd_sgd_static(fae_ctx *ctx, const fae_tables *hot_tables, float *const *h_hotW,
                                             const fae_batch *hot_batch, const float *gout, int64_t gout_row_stride,
                                             float lr)
{
    if (!ctx)
        return FAE_EINVAL;
    int32_t rc = fae_check_tables(ctx, hot_tables, "fae_embbag_bwd_sgd_static");
    if (rc != FAE_OK)
        return rc;
    rc = fae_check_batch(ctx, hot_tables, hot_batch, "fae_embbag_bwd_sgd_static");
    if (rc != FAE_OK)
        return rc;
    const size_t need = fae_bwd_workspace_bytes(hot_tables, hot_batch->n_samples, hot_batch->h_n_lookups);
    if (need == 0 || need > (size_t)FAE_BWD_STATIC_WS_BYTES)
        return fae_fail(ctx, FAE_ENOSPC,
                        "fae_embbag_bwd_sgd_static: this batch needs %zu bytes of workspace, the built-in one has %zu; "
                        "use fae_embbag_bwd_sgd with a workspace of the caller's",
                        need, (size_t)FAE_BWD_STATIC_WS_BYTES);
    if (!ctx->bwd_scratch) // resolved by fae_create; a context made before that is possible resolves it here
    {
        FAE_HIP(ctx, hipSetDevice(ctx->device));
        rc = fae_bwd_scratch_resolve(ctx, ctx->device, &ctx->bwd_scratch);
        if (rc != FAE_OK)
            return rc;
    }
    return fae_embbag_bwd_sgd(ctx, hot_tables, h_hotW, hot_batch, gout, gout_row_stride, lr, nullptr,
                              ctx->bwd_scratch, (size_t)FAE_BWD_STATIC_WS_BYTES);
}
