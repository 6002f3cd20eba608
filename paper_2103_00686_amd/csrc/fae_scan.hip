// Small shared device utilities: in-place exclusive scan of an int32 array by one
// workgroup, and a fill kernel (used instead of memset nodes so that every call
// stays capturable in a HIP graph).
#include "fae_internal.h"

__global__ __launch_bounds__(1024) void fae_scan_kernel(int32_t *data, int64_t n)
{
    __shared__ int lds[1024 / FAE_WAVE + 1];
    int carry = 0;
    for (int64_t base = 0; base < n; base += 4096) {
        const int64_t i0 = base + (int64_t)threadIdx.x * 4;
        int v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            v[k] = (i0 + k < n) ? data[i0 + k] : 0;
        int total;
        int ex = fae_block_excl_scan<1024>(v[0] + v[1] + v[2] + v[3], lds, &total);
        int run = carry + ex;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i0 + k < n)
                data[i0 + k] = run;
            run += v[k];
        }
        carry += total;
    }
    if (threadIdx.x == 0)
        data[n] = carry;
}

// data[0..n) -> exclusive prefix sums in place, data[n] = total (n+1 entries needed)
int32_t fae_scan_i32(fae_ctx *ctx, int32_t *data, int64_t n)
{
    fae_ktimer kt(ctx, FAE_K_OTHER);
    FAE_LAUNCH(ctx, fae_scan_kernel, dim3(1), dim3(1024), 0, ctx->stream, data, n);
    FAE_LAUNCH_CHECK(ctx);
    return FAE_OK;
}

__global__ __launch_bounds__(256) void fae_fill_kernel(uint32_t *p, int64_t n, uint32_t v)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (; i < n; i += stride)
        p[i] = v;
}

// ---------------------------------------------------------------------------------
// Plain streaming kernels: what a bandwidth-bound kernel reaches on this device, and
// transfers of known size against which hardware byte counters are scaled.  16 bytes
// per lane and access; a workgroup of 256 lanes owns chunks of U * 256 consecutive
// vectors (U accesses in flight per lane).  The grid is either one workgroup per chunk
// (the default: the dispatcher hands out short workgroups as fast as they retire,
// which measured best here) or a fixed number of workgroups per compute unit that
// stride over the chunks.  NT: non-temporal loads / stores.
// ---------------------------------------------------------------------------------
typedef float fae_probe_v4 __attribute__((ext_vector_type(4)));

template <int NT> __device__ __forceinline__ fae_probe_v4 probe_load(const fae_probe_v4 *p)
{
    if (NT)
        return __builtin_nontemporal_load(p);
    return *p;
}
template <int NT> __device__ __forceinline__ void probe_store(fae_probe_v4 *p, const fae_probe_v4 &v)
{
    if (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

template <int U, int NT>
__global__ __launch_bounds__(256) void fae_copy_probe_kernel(fae_probe_v4 *dst, const fae_probe_v4 *src, int64_t n)
{
    const int64_t chunk = (int64_t)U * 256;
    for (int64_t base = (int64_t)blockIdx.x * chunk; base < n; base += (int64_t)gridDim.x * chunk) {
        fae_probe_v4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256 + threadIdx.x;
            if (i < n)
                v[u] = probe_load<NT>(src + i);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256 + threadIdx.x;
            if (i < n)
                probe_store<NT>(dst + i, v[u]);
        }
    }
}

template <int U, int NT>
__global__ __launch_bounds__(256) void fae_read_probe_kernel(const fae_probe_v4 *src, int64_t n, float *sink)
{
    const int64_t chunk = (int64_t)U * 256;
    fae_probe_v4 s = {0.f, 0.f, 0.f, 0.f};
    for (int64_t base = (int64_t)blockIdx.x * chunk; base < n; base += (int64_t)gridDim.x * chunk) {
        fae_probe_v4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256 + threadIdx.x;
            v[u] = i < n ? probe_load<NT>(src + i) : s * 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            s += v[u];
    }
    if ((s.x + s.y) + (s.z + s.w) == 1.2345678e-30f) // never, for the buffers this is run on: keeps the loads alive
        sink[0] = s.x;
}

template <int U, int NT> __global__ __launch_bounds__(256) void fae_fill_probe_kernel(fae_probe_v4 *dst, int64_t n, float val)
{
    const int64_t chunk = (int64_t)U * 256;
    const fae_probe_v4 v = {val, val, val, val};
    for (int64_t base = (int64_t)blockIdx.x * chunk; base < n; base += (int64_t)gridDim.x * chunk) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256 + threadIdx.x;
            if (i < n)
                probe_store<NT>(dst + i, v);
        }
    }
}

namespace {
// the launch shape of a probe: the context's probe_* options, or the shape that measured best
struct ProbeShape {
    int unroll, nt;
    unsigned grid;
};
ProbeShape probe_shape(const fae_ctx *ctx, int64_t n, int best_unroll, int best_nt)
{
    ProbeShape p;
    p.unroll = ctx->opt_probe_unroll ? (int)ctx->opt_probe_unroll : best_unroll;
    p.nt = ctx->opt_probe_nt >= 0 ? (int)ctx->opt_probe_nt : best_nt;
    int64_t blocks = (n + (int64_t)p.unroll * 256 - 1) / ((int64_t)p.unroll * 256);
    if (ctx->opt_probe_wgs_per_cu > 0 && blocks > ctx->opt_probe_wgs_per_cu * ctx->n_cu)
        blocks = ctx->opt_probe_wgs_per_cu * ctx->n_cu;
    if (blocks > 2147483647LL)
        blocks = 2147483647LL; // the chunks beyond are reached by the stride
    p.grid = (unsigned)blocks;
    return p;
}
#define PROBE_DISPATCH(KERNEL, shape, ...)                                                                   \
    do {                                                                                                     \
        const dim3 g_((shape).grid), b_(256);                                                                \
        switch ((shape).unroll * 2 + (shape).nt) {                                                           \
        case 2: FAE_LAUNCH(ctx, (KERNEL<1, 0>), g_, b_, 0, ctx->stream, __VA_ARGS__); break;              \
        case 3: FAE_LAUNCH(ctx, (KERNEL<1, 1>), g_, b_, 0, ctx->stream, __VA_ARGS__); break;              \
        case 4: FAE_LAUNCH(ctx, (KERNEL<2, 0>), g_, b_, 0, ctx->stream, __VA_ARGS__); break;              \
        case 5: FAE_LAUNCH(ctx, (KERNEL<2, 1>), g_, b_, 0, ctx->stream, __VA_ARGS__); break;              \
        case 8: FAE_LAUNCH(ctx, (KERNEL<4, 0>), g_, b_, 0, ctx->stream, __VA_ARGS__); break;              \
        case 9: FAE_LAUNCH(ctx, (KERNEL<4, 1>), g_, b_, 0, ctx->stream, __VA_ARGS__); break;              \
        case 16: FAE_LAUNCH(ctx, (KERNEL<8, 0>), g_, b_, 0, ctx->stream, __VA_ARGS__); break;             \
        default: FAE_LAUNCH(ctx, (KERNEL<8, 1>), g_, b_, 0, ctx->stream, __VA_ARGS__); break;             \
        }                                                                                                    \
    } while (0)
} // namespace

extern "C" int32_t fae_read_probe(fae_ctx *ctx, const void *src, size_t bytes, float *sink)
{
    if (!ctx || !src || !sink || bytes % 16 != 0 || ((uintptr_t)src) % 16 != 0)
        return fae_fail(ctx, FAE_EINVAL, "fae_read_probe: null or misaligned argument");
    const int64_t n = (int64_t)(bytes / 16);
    if (n == 0)
        return FAE_OK;
    const ProbeShape shape = probe_shape(ctx, n, 4, 1);
    fae_ktimer kt(ctx, FAE_K_READ_PROBE);
    PROBE_DISPATCH(fae_read_probe_kernel, shape, (const fae_probe_v4 *)src, n, sink);
    FAE_LAUNCH_CHECK(ctx);
    return FAE_OK;
}

extern "C" int32_t fae_copy_probe(fae_ctx *ctx, void *dst, const void *src, size_t bytes)
{
    if (!ctx || !dst || !src || bytes % 16 != 0 || ((uintptr_t)dst) % 16 != 0 || ((uintptr_t)src) % 16 != 0)
        return fae_fail(ctx, FAE_EINVAL, "fae_copy_probe: null or misaligned argument");
    const int64_t n = (int64_t)(bytes / 16);
    if (n == 0)
        return FAE_OK;
    const ProbeShape shape = probe_shape(ctx, n, 1, 0);
    fae_ktimer kt(ctx, FAE_K_COPY_PROBE);
    PROBE_DISPATCH(fae_copy_probe_kernel, shape, (fae_probe_v4 *)dst, (const fae_probe_v4 *)src, n);
    FAE_LAUNCH_CHECK(ctx);
    return FAE_OK;
}

extern "C" int32_t fae_fill_probe(fae_ctx *ctx, void *dst, size_t bytes, float value)
{
    if (!ctx || !dst || bytes % 16 != 0 || ((uintptr_t)dst) % 16 != 0)
        return fae_fail(ctx, FAE_EINVAL, "fae_fill_probe: null or misaligned argument");
    const int64_t n = (int64_t)(bytes / 16);
    if (n == 0)
        return FAE_OK;
    const ProbeShape shape = probe_shape(ctx, n, 1, 0);
    fae_ktimer kt(ctx, FAE_K_FILL_PROBE);
    PROBE_DISPATCH(fae_fill_probe_kernel, shape, (fae_probe_v4 *)dst, n, value);
    FAE_LAUNCH_CHECK(ctx);
    return FAE_OK;
}

int32_t fae_fill_u32(fae_ctx *ctx, void *p, int64_t n_words, uint32_t v)
{
    return fae_fill_u32_on(ctx, ctx->stream, p, n_words, v);
}

int32_t fae_fill_u32_on(fae_ctx *ctx, hipStream_t st, void *p, int64_t n_words, uint32_t v)
{
    if (n_words <= 0)
        return FAE_OK;
    int64_t blocks = (n_words + 255) / 256;
    if (blocks > 65536)
        blocks = 65536;
    fae_ktimer kt(ctx, FAE_K_FILL, st);
    FAE_LAUNCH(ctx, fae_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (uint32_t *)p, n_words, v);
    FAE_LAUNCH_CHECK(ctx);
    return FAE_OK;
}
