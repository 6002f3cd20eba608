// Context, error reporting and argument validation of libfae.
#include <stdarg.h>
#include <stdlib.h>

#include <new>

#include "fae_internal.h"

int32_t fae_fail(fae_ctx *ctx, int32_t code, const char *fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

__global__ void fae_clear_words_kernel(uint32_t *p, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        p[i] = 0u;
}

static bool fae_make_side_streams(fae_ctx *ctx)
{
    for (int i = 0; i < fae_ctx::N_AUX; ++i)
        if (hipStreamCreateWithFlags(&ctx->aux_stream[i], hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&ctx->ev_fork[i], hipEventDisableTiming) != hipSuccess)
            return false;
    return true;
}

static bool fae_make_join_events(fae_ctx *ctx)
{
    for (auto &e : ctx->presort)
        if (hipEventCreateWithFlags(&e.ev_join, hipEventDisableTiming) != hipSuccess)
            return false;
    return true;
}

extern "C" int32_t fae_create(fae_ctx **out, int32_t device, void *hip_stream)
{
    if (!out)
        return FAE_EINVAL;
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev)
        return FAE_EHIP;
    fae_ctx *ctx = new (std::nothrow) fae_ctx();
    if (!ctx)
        return FAE_ENOSPC;
    ctx->device = device;
    ctx->stream = (hipStream_t)hip_stream;
    if (hipSetDevice(device) != hipSuccess) {
        delete ctx;
        return FAE_EHIP;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) {
        delete ctx;
        return FAE_EHIP;
    }
    ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    if (hipMalloc((void **)&ctx->d_block, FAE_BLK_WORDS * sizeof(uint32_t)) != hipSuccess) {
        delete ctx;
        return FAE_EHIP;
    }
    if (hipHostMalloc((void **)&ctx->h_block, FAE_BLK_WORDS * sizeof(uint32_t), hipHostMallocDefault) !=
        hipSuccess) {
        (void)hipFree(ctx->d_block);
        delete ctx;
        return FAE_EHIP;
    }
    memset(ctx->h_block, 0, FAE_BLK_WORDS * sizeof(uint32_t));
    // the built-in backward workspace of this device (the device is current here)
    if (fae_bwd_scratch_resolve(ctx, device, &ctx->bwd_scratch) != FAE_OK) {
        (void)hipFree(ctx->d_block);
        (void)hipHostFree(ctx->h_block);
        delete ctx;
        return FAE_EHIP;
    }
    if (!fae_make_side_streams(ctx) || !fae_make_join_events(ctx)) {
        (void)hipFree(ctx->d_block);
        (void)hipHostFree(ctx->h_block);
        delete ctx;
        return FAE_EHIP;
    }
    FAE_LAUNCH(ctx, fae_clear_words_kernel, dim3(FAE_BLK_WORDS / 256), dim3(256), 0, ctx->stream,
                       ctx->d_block, FAE_BLK_WORDS);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(ctx->stream) != hipSuccess) {
        (void)hipFree(ctx->d_block);
        (void)hipHostFree(ctx->h_block);
        delete ctx;
        return FAE_EHIP;
    }
    *out = ctx;
    return FAE_OK;
}

extern "C" void fae_destroy(fae_ctx *ctx)
{
    if (!ctx)
        return;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    for (int i = 0; i < fae_ctx::N_AUX; ++i) {
        if (ctx->aux_stream[i]) {
            (void)hipStreamSynchronize(ctx->aux_stream[i]);
            (void)hipStreamDestroy(ctx->aux_stream[i]);
        }
        if (ctx->ev_fork[i])
            (void)hipEventDestroy(ctx->ev_fork[i]);
    }
    for (auto &e : ctx->presort)
        if (e.ev_join)
            (void)hipEventDestroy(e.ev_join);
    for (const fae_timed_launch &t : ctx->timed) {
        (void)hipEventDestroy(t.e0);
        (void)hipEventDestroy(t.e1);
    }
    for (hipEvent_t e : ctx->event_pool)
        (void)hipEventDestroy(e);
    (void)hipFree(ctx->d_block);
    (void)hipHostFree(ctx->h_block);
    delete ctx;
}

// ---------------------------------------------------------------------------------
// per-kernel timing
// ---------------------------------------------------------------------------------
static hipEvent_t take_event(fae_ctx *c)
{
    if (!c->event_pool.empty()) {
        hipEvent_t e = c->event_pool.back();
        c->event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess)
        return nullptr;
    return e;
}

bool fae_timing_begin(fae_ctx *ctx, hipEvent_t *e0, hipEvent_t *e1)
{
    if (!ctx || !ctx->timing)
        return false;
    *e0 = take_event(ctx);
    *e1 = take_event(ctx);
    if (*e0 && *e1)
        return true;
    if (*e0)
        ctx->event_pool.push_back(*e0);
    if (*e1)
        ctx->event_pool.push_back(*e1);
    return false;
}

void fae_timing_end(fae_ctx *ctx, hipEvent_t e0, hipEvent_t e1)
{
    fae_timed_launch t;
    t.id = ctx->cur_class;
    t.e0 = e0;
    t.e1 = e1;
    ctx->timed.push_back(t);
}

static int32_t timing_collect(fae_ctx *ctx)
{
    FAE_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (int i = 0; i < fae_ctx::N_AUX; ++i)
        FAE_HIP(ctx, hipStreamSynchronize(ctx->aux_stream[i]));
    for (const fae_timed_launch &t : ctx->timed) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t.e0, t.e1) == hipSuccess) {
            ctx->t_total_ms[t.id] += ms;
            ctx->t_launches[t.id] += 1;
        }
        ctx->event_pool.push_back(t.e0);
        ctx->event_pool.push_back(t.e1);
    }
    ctx->timed.clear();
    return FAE_OK;
}

extern "C" int32_t fae_timing_enable(fae_ctx *ctx, int32_t on)
{
    if (!ctx)
        return FAE_EINVAL;
    int32_t rc = timing_collect(ctx);
    ctx->timing = on != 0;
    return rc;
}

extern "C" int32_t fae_timing_reset(fae_ctx *ctx)
{
    if (!ctx)
        return FAE_EINVAL;
    int32_t rc = timing_collect(ctx);
    for (int i = 0; i < FAE_K_COUNT; ++i) {
        ctx->t_total_ms[i] = 0.0;
        ctx->t_launches[i] = 0;
    }
    return rc;
}

extern "C" int32_t fae_timing_read(fae_ctx *ctx, int32_t kernel_class, double *h_total_ms, int64_t *h_launches)
{
    if (!ctx || kernel_class < 0 || kernel_class >= FAE_K_COUNT || !h_total_ms || !h_launches)
        return FAE_EINVAL;
    int32_t rc = timing_collect(ctx);
    *h_total_ms = ctx->t_total_ms[kernel_class];
    *h_launches = ctx->t_launches[kernel_class];
    return rc;
}

extern "C" const char *fae_kernel_name(int32_t k)
{
    static const char *names[FAE_K_COUNT] = {"fwd",        "bwd_keys",  "sort_hist", "sort_colscan", "sort_scatter",
                                             "bwd_reduce", "bwd_fixup", "lds_sort",  "fill",         "profile",
                                             "partition",  "build",     "other",     "copy_probe",
                                             "fwd_sort",   "sync_rows", "estimate",  "read_probe",
                                             "fill_probe"};
    return (k >= 0 && k < FAE_K_COUNT) ? names[k] : "?";
}

extern "C" const char *fae_last_error(const fae_ctx *ctx) { return ctx ? ctx->err : "null context"; }

extern "C" const char *fae_version(void) { return "libfae 0.1 (gfx950)"; }

extern "C" int32_t fae_set_option(fae_ctx *ctx, const char *name, int64_t value)
{
    if (!ctx || !name)
        return FAE_EINVAL;
    if (!strcmp(name, "profile_variant") && value >= 0 && value <= 2)
        ctx->opt_profile = value;
    else if (!strcmp(name, "fwd_variant") && value >= 0 && value <= 2)
        ctx->opt_fwd = value;
    else if (!strcmp(name, "sort_variant") && value >= 0 && value <= 4)
        ctx->opt_sort = value;
    else if (!strcmp(name, "sort_order") && value >= 0 && value <= 1)
        ctx->opt_sort_order = value;
    else if (!strcmp(name, "fwd_stream_out") && value >= 0 && value <= 1)
        ctx->opt_fwd_stream = value;
    else if (!strcmp(name, "reduce_span") && (value == 0 || value == 64 || value == 128 || value == 256))
        ctx->opt_span = value;
    else if (!strcmp(name, "fixup_variant") && value >= 0 && value <= 1)
        ctx->opt_fixup = value;
    else if (!strcmp(name, "reduce_variant") && value >= 0 && value <= 2)
        ctx->opt_reduce = value;
    else if (!strcmp(name, "reduce_wg_waves") && (value == 0 || value == 1 || value == 2 || value == 4))
        ctx->opt_wg_waves = value;
    else if (!strcmp(name, "reduce_unroll") && (value == 0 || value == 2 || value == 4 || value == 8))
        ctx->opt_unroll = value;
    else if (!strcmp(name, "handoff_fences") && value >= 0 && value <= 1)
        ctx->opt_handoff = value;
    else if (!strcmp(name, "probe_unroll") && (value == 0 || value == 1 || value == 2 || value == 4 || value == 8))
        ctx->opt_probe_unroll = value;
    else if (!strcmp(name, "probe_nt") && value >= -1 && value <= 1)
        ctx->opt_probe_nt = value;
    else if (!strcmp(name, "probe_wgs_per_cu") && value >= 0 && value <= 64)
        ctx->opt_probe_wgs_per_cu = value;
    else
        return fae_fail(ctx, FAE_EINVAL, "fae_set_option: unknown option or value: %s=%lld", name,
                        (long long)value);
    return FAE_OK;
}

int32_t fae_readback(fae_ctx *ctx, int first, int n)
{
    FAE_HIP(ctx, hipMemcpyAsync(ctx->h_block + first, ctx->d_block + first, (size_t)n * sizeof(uint32_t),
                                hipMemcpyDeviceToHost, ctx->stream));
    FAE_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return FAE_OK;
}

int32_t fae_sync_status(fae_ctx *ctx)
{
    for (int i = 0; i < fae_ctx::N_AUX; ++i)
        if (ctx->aux_stream[i])
            FAE_HIP(ctx, hipStreamSynchronize(ctx->aux_stream[i]));
    int32_t rc = fae_readback(ctx, FAE_BLK_STATUS, 1);
    if (rc != FAE_OK)
        return rc;
    uint32_t st = ctx->h_block[FAE_BLK_STATUS];
    if (st == 0)
        return FAE_OK;
    FAE_LAUNCH(ctx, fae_clear_words_kernel, dim3(1), dim3(64), 0, ctx->stream, ctx->d_block, 1);
    FAE_LAUNCH_CHECK(ctx);
    FAE_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (st & FAE_STATUS_EINTERNAL)
        return fae_fail(ctx, FAE_EHIP, "internal: a bounded wait inside a kernel gave up; results of that call are invalid");
    if (st & FAE_STATUS_ERANGE)
        return fae_fail(ctx, FAE_ERANGE, "device detected an index/slot out of range or a malformed CSR");
    return fae_fail(ctx, FAE_ENOSPC, "device detected an output capacity overflow");
}

extern "C" int32_t fae_sync(fae_ctx *ctx)
{
    if (!ctx)
        return FAE_EINVAL;
    return fae_sync_status(ctx);
}

int32_t fae_check_tables(fae_ctx *ctx, const fae_tables *t, const char *who)
{
    if (!ctx)
        return FAE_EINVAL;
    if (!t || !t->h_rows)
        return fae_fail(ctx, FAE_EINVAL, "%s: null tables", who);
    if (t->n_tables < 1 || t->n_tables > FAE_MAX_TABLES)
        return fae_fail(ctx, FAE_EINVAL, "%s: n_tables=%d outside [1,%d]", who, t->n_tables, FAE_MAX_TABLES);
    if (t->dim < 1 || t->dim > 65536)
        return fae_fail(ctx, FAE_EINVAL, "%s: dim=%d outside [1,65536]", who, t->dim);
    for (int z = 0; z < t->n_tables; ++z)
        if (t->h_rows[z] < 0 || t->h_rows[z] >= 2147483647LL)
            return fae_fail(ctx, FAE_EINVAL, "%s: rows[%d]=%lld outside [0,2^31-1)", who, z,
                            (long long)t->h_rows[z]);
    return FAE_OK;
}

int32_t fae_check_batch(fae_ctx *ctx, const fae_tables *t, const fae_batch *b, const char *who)
{
    if (!b || !b->h_indices || !b->h_n_lookups)
        return fae_fail(ctx, FAE_EINVAL, "%s: null batch", who);
    if (b->n_samples < 0 || b->n_samples >= 2147483647LL)
        return fae_fail(ctx, FAE_EINVAL, "%s: n_samples=%lld outside [0,2^31-1)", who, (long long)b->n_samples);
    if (b->index_bits != 0 && b->index_bits != 32 && b->index_bits != 64)
        return fae_fail(ctx, FAE_EINVAL, "%s: index_bits=%d is neither 32 nor 64", who, b->index_bits);
    for (int z = 0; z < t->n_tables; ++z) {
        int64_t nl = b->h_n_lookups[z];
        if (nl < 0 || nl >= 2147483647LL)
            return fae_fail(ctx, FAE_EINVAL, "%s: n_lookups[%d]=%lld outside [0,2^31-1)", who, z, (long long)nl);
        bool one_hot = !b->h_offsets || !b->h_offsets[z];
        if (one_hot && nl != b->n_samples)
            return fae_fail(ctx, FAE_EINVAL, "%s: table %d has no offsets but n_lookups != n_samples", who, z);
        if (nl > 0 && !b->h_indices[z])
            return fae_fail(ctx, FAE_EINVAL, "%s: null indices for table %d", who, z);
    }
    return FAE_OK;
}
