// Internal declarations shared by the translation units of libfae (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "../../include/fae.h"

// ---------------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------------
#define FAE_STATUS_ERANGE 1u
#define FAE_STATUS_ENOSPC 2u
#define FAE_STATUS_EINTERNAL 4u // a bounded wait inside a kernel gave up

// word offsets inside the 4 KiB device / pinned-host blocks
#define FAE_BLK_STATUS 0
#define FAE_BLK_SCALARS 64 // first word usable for scalar read-backs
#define FAE_BLK_WORDS 1024

struct fae_timed_launch {
    int id;
    hipEvent_t e0, e1;
};

struct fae_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    uint32_t *d_block = nullptr; // device, FAE_BLK_WORDS words
    uint32_t *h_block = nullptr; // pinned host mirror
    int n_cu = 256;
    int64_t opt_profile = 0; // 0 auto, 1 global atomics, 2 LDS-privatised
    int64_t opt_fwd = 0;     // 0 auto, 1 group-per-bag, 2 wave-per-bag
    int64_t opt_sort = 0;    // 0 auto, 1 global radix, 2 LDS per table
    int64_t opt_sort_order = 0; // LDS sort: 0 stable (lookups of a slot in batch order), 1 counting sort (any order)
    int64_t opt_fwd_stream = 1; // non-temporal stores for the pooled output
    int64_t opt_span = 0;       // lookups per wave in the reduce kernel (0 = auto)
    int64_t opt_fixup = 0;      // runs that cross span borders: 0 auto (inside the reduce kernel), 1 separate kernel
    int64_t opt_reduce = 0;     // reduce kernel: 0 auto, 1 scan across lane groups, 2 a share of the span per lane group
    int64_t opt_wg_waves = 0;   // reduce kernel: waves per workgroup (0 = auto, 1, 2, 4)
    int64_t opt_unroll = 0;     // gradient rows in flight per lane group in the second form (0 = auto, 4, 8)
    int64_t opt_handoff = 0;    // border sums between workgroups: 0 auto (device-scope accesses, wave-level ordering), 1 device-scope fences
    // launch shape of the streaming probes (0 / -1: the shape that measured best)
    int64_t opt_probe_unroll = 0;      // 16-byte accesses in flight per lane: 1, 2, 4, 8
    int64_t opt_probe_nt = -1;         // non-temporal accesses: 0, 1
    int64_t opt_probe_wgs_per_cu = 0;  // 0: one workgroup per chunk; n: n workgroups per compute unit striding over the chunks
    char err[512] = {0};
    // device address of this device's copy of the library's built-in backward workspace
    // (fae_embbag_bwd_sgd_static); resolved by fae_create
    void *bwd_scratch = nullptr;
    // side stream for work that may overlap the main stream (backward presort)
    // two of them, taken in turn: the sorts of consecutive batches may overlap each other
    static constexpr int N_AUX = 2;
    hipStream_t aux_stream[N_AUX] = {nullptr, nullptr};
    hipEvent_t ev_fork[N_AUX] = {nullptr, nullptr};
    int aux_next = 0;
    // Sorted (slot, sample) pairs waiting for their backward call, one entry per workspace: a
    // caller may sort the next batch (into a second workspace) while this one is still in use.
    static constexpr int N_PRESORT = 4;
    struct Presort {
        bool valid = false;
        bool side = false; // sorted on the side stream (needs the join event) or on the main stream
        const void *ws = nullptr;
        // the batch the pairs were sorted from: every table's index and offset buffers and its lookups
        int n_tables = 0;
        const void *indices[FAE_MAX_TABLES] = {nullptr};
        const void *offsets[FAE_MAX_TABLES] = {nullptr};
        int64_t n_lookups_z[FAE_MAX_TABLES] = {0};
        int64_t n_samples = 0;
        int cur = 0;
        uint64_t age = 0;
        hipEvent_t ev_join = nullptr;
    } presort[N_PRESORT];
    uint64_t presort_clock = 0;
    // the entry that holds (or will hold) the pairs in workspace ws: the one already bound to it,
    // else a free one, else the oldest (whose owner then has to wait for it: see the callers)
    Presort *presort_slot(const void *ws)
    {
        Presort *pick = &presort[0];
        for (auto &e : presort) {
            if (e.valid && e.ws == ws)
                return &e;
            if (pick->valid && (!e.valid || e.age < pick->age))
                pick = &e;
        }
        return pick;
    }
    Presort *presort_find(const void *ws)
    {
        for (auto &e : presort)
            if (e.valid && e.ws == ws)
                return &e;
        return nullptr;
    }
    // Remember which batch the pairs in e's workspace belong to / ask whether b is that batch.  A
    // batch is known by the buffers it names: the same pointers and sizes for every table.  (A
    // caller that rewrites a buffer in place between the sort and the backward is outside what
    // the pointers can tell: the batch and the workspace must stay untouched in between.)
    static void presort_bind(Presort *e, int nt, const fae_batch *b)
    {
        e->n_tables = nt;
        e->n_samples = b->n_samples;
        for (int z = 0; z < nt; ++z) {
            e->indices[z] = b->h_indices[z];
            e->offsets[z] = b->h_offsets ? b->h_offsets[z] : nullptr;
            e->n_lookups_z[z] = b->h_n_lookups[z];
        }
    }
    static bool presort_is(const Presort *e, int nt, const fae_batch *b)
    {
        if (e->n_tables != nt || e->n_samples != b->n_samples)
            return false;
        for (int z = 0; z < nt; ++z)
            if (e->indices[z] != b->h_indices[z] || e->offsets[z] != (b->h_offsets ? b->h_offsets[z] : nullptr) ||
                e->n_lookups_z[z] != b->h_n_lookups[z])
                return false;
        return true;
    }
    // per-kernel timing
    bool timing = false;
    int cur_class = FAE_K_OTHER;          // kernel class of the launches issued right now (set by fae_ktimer)
    std::vector<fae_timed_launch> timed;  // launches recorded since the last read
    std::vector<hipEvent_t> event_pool;   // events ready for reuse
    double t_total_ms[FAE_K_COUNT] = {0};
    int64_t t_launches[FAE_K_COUNT] = {0};
};

// Names the kernel class of the launches issued during its lifetime (for the per-kernel timing).
struct fae_ktimer {
    fae_ctx *c;
    int prev;
    fae_ktimer(fae_ctx *ctx, int id) : c(ctx), prev(ctx ? ctx->cur_class : 0)
    {
        if (c)
            c->cur_class = id;
    }
    fae_ktimer(fae_ctx *ctx, int id, hipStream_t) : fae_ktimer(ctx, id) {}
    ~fae_ktimer()
    {
        if (c)
            c->cur_class = prev;
    }
};

// With timing on: two events for one launch (false when timing is off or no event could be made);
// fae_timing_end files them under the current kernel class.
bool fae_timing_begin(fae_ctx *ctx, hipEvent_t *e0, hipEvent_t *e1);
void fae_timing_end(fae_ctx *ctx, hipEvent_t e0, hipEvent_t e1);

// Every kernel of the library is launched through this.  With timing on, the launch itself carries
// the two events, which the device stamps at the kernel's own start and end: the figure does not
// depend on whether the stream was idle, and holds nothing but the kernel.
#define FAE_LAUNCH(ctx, kernel, grid, block, shmem, stream, ...)                                          \
    do {                                                                                                  \
        hipEvent_t e0_ = nullptr, e1_ = nullptr;                                                          \
        if (fae_timing_begin((ctx), &e0_, &e1_)) {                                                        \
            hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, e0_, e1_, 0, __VA_ARGS__);          \
            fae_timing_end((ctx), e0_, e1_);                                                              \
        } else                                                                                            \
            hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                          \
    } while (0)

int32_t fae_fail(fae_ctx *ctx, int32_t code, const char *fmt, ...);
// fae_bwd.hip: device address of the built-in backward workspace on `device` (which is current)
int32_t fae_bwd_scratch_resolve(fae_ctx *ctx, int device, void **out);
// copy n words of the device block (from word `first`) to the pinned block and wait
int32_t fae_readback(fae_ctx *ctx, int first, int n);
// wait for the stream, fetch + clear the sticky status; maps it to an error code
int32_t fae_sync_status(fae_ctx *ctx);
int32_t fae_check_tables(fae_ctx *ctx, const fae_tables *t, const char *who);
int32_t fae_check_batch(fae_ctx *ctx, const fae_tables *t, const fae_batch *b, const char *who);
// data[0..n) -> exclusive prefix sums in place, data[n] = total (one workgroup; n+1 entries)
int32_t fae_scan_i32(fae_ctx *ctx, int32_t *data, int64_t n);
// fill n 32-bit words (a kernel, not a memset node: stays graph-capturable)
int32_t fae_fill_u32(fae_ctx *ctx, void *p, int64_t n_words, uint32_t v);
int32_t fae_fill_u32_on(fae_ctx *ctx, hipStream_t st, void *p, int64_t n_words, uint32_t v);

#define FAE_HIP(ctx, call)                                                                   \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess)                                                                \
            return fae_fail((ctx), FAE_EHIP, "%s: %s (%s:%d)", #call, hipGetErrorString(e_), \
                            __FILE__, __LINE__);                                             \
    } while (0)

#define FAE_LAUNCH_CHECK(ctx) FAE_HIP(ctx, hipGetLastError())

static inline size_t fae_align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// carve aligned sub-buffers out of a caller-provided workspace
struct fae_carver {
    char *base;
    size_t used;
    size_t cap;
    bool ok;
    fae_carver(void *ws, size_t bytes) : base((char *)ws), used(0), cap(bytes), ok(true) {}
    template <typename T> T *take(size_t n)
    {
        size_t b = fae_align_up(n * sizeof(T), 256);
        if (b == 0)
            b = 256;
        T *p = (T *)(base + used);
        used += b;
        if (used > cap || base == nullptr)
            ok = false;
        return p;
    }
};

// ---------------------------------------------------------------------------------
// device helpers (wave64)
// ---------------------------------------------------------------------------------
#ifdef __HIPCC__

#define FAE_WAVE 64

__device__ __forceinline__ int fae_lane() { return (int)__lane_id(); }

__device__ __forceinline__ void fae_flag(uint32_t *status, uint32_t bit)
{
    // sticky status word; plain OR through a vector atomic, rare path
    atomicOr(status + FAE_BLK_STATUS, bit);
}

// table that owns flat block index b, given exclusive prefix blk_start[0..nt] (an array of
// FAE_MAX_TABLES + 1 entries in the kernel's arguments).  The prefix is non-decreasing, so the
// owner is the number of tables that start at or before b.  Counted in two rounds of seven
// independent loads each (every eighth entry, then the entries of the group of eight found; one
// round for up to eight tables):
// a search that walks up to the owner is a chain of dependent loads as long as the table's
// number, which the workgroups of the last tables pay in full before their first useful load.
__device__ __forceinline__ int fae_find_table(const int32_t *blk_start, int nt, int b)
{
    static_assert(FAE_MAX_TABLES == 64, "two levels of eight");
    if (nt <= 1)
        return 0;
    int v[8]; // every load of a round is issued whatever the others return (the array has an entry for every index)
    int base = 0;
    if (nt > 8) {
#pragma unroll
        for (int i = 1; i < 8; ++i)
            v[i] = blk_start[8 * i];
#pragma unroll
        for (int i = 1; i < 8; ++i)
            base += ((8 * i < nt) & (b >= v[i])) ? 8 : 0;
    }
#pragma unroll
    for (int i = 1; i < 8; ++i)
        v[i] = blk_start[base + i];
    int z = base;
#pragma unroll
    for (int i = 1; i < 8; ++i)
        z += ((base + i < nt) & (b >= v[i])) ? 1 : 0;
    return z;
}

// raw row id j of an index array that holds int32 or int64 values; -1 if it is outside [0, rows)
__device__ __forceinline__ int fae_load_row(const void *idx, int64_t j, int wide, int rows)
{
    if (wide) {
        const int64_t v = ((const int64_t *)idx)[j];
        return (v >= 0 && v < (int64_t)rows) ? (int)v : -1;
    }
    const int v = ((const int32_t *)idx)[j];
    return (unsigned)v < (unsigned)rows ? v : -1;
}

// inclusive scan across the 64 lanes of a wave
__device__ __forceinline__ int fae_wave_incl_scan(int v)
{
    int lane = fae_lane();
#pragma unroll
    for (int d = 1; d < FAE_WAVE; d <<= 1) {
        int n = __shfl_up(v, d, FAE_WAVE);
        if (lane >= d)
            v += n;
    }
    return v;
}

// exclusive scan across a block of BLOCK threads (BLOCK multiple of 64, <= 1024).
// lds must hold BLOCK/64 + 1 ints.  Returns the exclusive prefix; *total = block sum.
// Every thread adds up the wave totals itself (at most sixteen LDS reads of the same addresses,
// issued together): no thread does it for the others while they wait at a third barrier.
template <int BLOCK> __device__ __forceinline__ int fae_block_excl_scan(int v, int *lds, int *total)
{
    constexpr int NW = BLOCK / FAE_WAVE;
    int lane = fae_lane(), w = threadIdx.x / FAE_WAVE;
    int inc = fae_wave_incl_scan(v);
    __syncthreads(); // lds may still be read from a previous call
    if (lane == FAE_WAVE - 1)
        lds[w] = inc;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const int t = lds[i];
        all += t;
        before += i < w ? t : 0;
    }
    *total = all;
    return before + inc - v;
}

// first position in sorted a[lo,hi) whose value is > key (upper bound)
__device__ __forceinline__ int fae_upper_bound(const int32_t *a, int lo, int hi, int key)
{
    while (lo < hi) {
        int mid = lo + ((hi - lo) >> 1);
        if (a[mid] <= key)
            lo = mid + 1;
        else
            hi = mid;
    }
    return lo;
}

// sample that owns lookup j in CSR offsets[0..n_samples] (offsets[s] <= j < offsets[s+1])
__device__ __forceinline__ int fae_sample_of(const int32_t *offsets, int n_samples, int j)
{
    int s = fae_upper_bound(offsets, 0, n_samples + 1, j) - 1;
    return s < 0 ? 0 : (s >= n_samples ? n_samples - 1 : s); // in range even for a malformed CSR
}

#endif // __HIPCC__
