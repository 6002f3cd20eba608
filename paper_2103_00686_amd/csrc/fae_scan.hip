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
    hipLaunchKernelGGL(fae_scan_kernel, dim3(1), dim3(1024), 0, ctx->stream, data, n);
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

__global__ __launch_bounds__(256) void fae_copy_probe_kernel(float4 *dst, const float4 *src, int64_t n)
{
    // four independent 16-byte loads per lane in flight, then four stores
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const float4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a;
        dst[i + stride] = b;
        dst[i + 2 * stride] = c;
        dst[i + 3 * stride] = d;
    }
    for (; i < n; i += stride)
        dst[i] = src[i];
}

__global__ __launch_bounds__(256) void fae_read_probe_kernel(const float4 *src, int64_t n, float *sink)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (; i + 3 * stride < n; i += 4 * stride) {
        const float4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        s.x += (a.x + b.x) + (c.x + d.x);
        s.y += (a.y + b.y) + (c.y + d.y);
        s.z += (a.z + b.z) + (c.z + d.z);
        s.w += (a.w + b.w) + (c.w + d.w);
    }
    for (; i < n; i += stride) {
        const float4 a = src[i];
        s.x += a.x;
        s.y += a.y;
        s.z += a.z;
        s.w += a.w;
    }
    if ((s.x + s.y) + (s.z + s.w) == 1.2345678e-30f)
        sink[0] = s.x;
}

extern "C" int32_t fae_read_probe(fae_ctx *ctx, const void *src, size_t bytes, float *sink)
{
    if (!ctx || !src || !sink || bytes % 16 != 0 || ((uintptr_t)src) % 16 != 0)
        return fae_fail(ctx, FAE_EINVAL, "fae_read_probe: null or misaligned argument");
    const int64_t n = (int64_t)(bytes / 16);
    if (n == 0)
        return FAE_OK;
    int64_t blocks = (n + 255) / 256;
    const int64_t cap = (int64_t)ctx->n_cu * 32;
    if (blocks > cap)
        blocks = cap;
    fae_ktimer kt(ctx, FAE_K_READ_PROBE);
    hipLaunchKernelGGL(fae_read_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, (const float4 *)src, n,
                       sink);
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
    int64_t blocks = (n + 255) / 256;
    const int64_t cap = (int64_t)ctx->n_cu * 32; // grid-stride: a few waves per SIMD, many vectors per lane
    if (blocks > cap)
        blocks = cap;
    fae_ktimer kt(ctx, FAE_K_COPY_PROBE);
    hipLaunchKernelGGL(fae_copy_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, (float4 *)dst,
                       (const float4 *)src, n);
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
    hipLaunchKernelGGL(fae_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (uint32_t *)p, n_words, v);
    FAE_LAUNCH_CHECK(ctx);
    return FAE_OK;
}
