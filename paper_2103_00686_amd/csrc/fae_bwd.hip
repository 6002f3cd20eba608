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
// No float atomics: every row has exactly one writer and a fixed summation order.
// Bandwidth bound: per lookup one gradient row is read, per distinct row one weight
// row is read and written; the sort moves 16 B per lookup and pass.
#include "fae_internal.h"
#include "fae_device.h"

// ---------------------------------------------------------------------------------
// sort geometry
// ---------------------------------------------------------------------------------
#define SORT_THREADS 256
#define SORT_ITEMS 16
#define SORT_WAVES (SORT_THREADS / FAE_WAVE)
#define SORT_TILE (SORT_THREADS * SORT_ITEMS)
// short lists: smaller tiles, so that a chained pass has enough workgroups and a short chain per tile
#define SORT_ITEMS_SMALL 4
#define SORT_TILE_SMALL (SORT_THREADS * SORT_ITEMS_SMALL)
#define SORT_SMALL_MAX_TILES 1024 // small tiles are used up to this many of them

#define BWD_SPAN_MAX 256 // sorted lookups per wave in the reduce kernel (multiple of 64)
#define BWD_SPAN_MIN 64
#define DBG_TILE 2048

struct BwdArgs {
    float *W[FAE_MAX_TABLES];
    const int32_t *slots[FAE_MAX_TABLES];
    const int32_t *offsets[FAE_MAX_TABLES];
    int32_t n_hot[FAE_MAX_TABLES];
    int32_t seg_start[FAE_MAX_TABLES + 1];  // prefix of lookups per table
    int32_t blk_start[FAE_MAX_TABLES + 1];  // prefix of workgroups per table (kernel specific)
    int32_t tile_start[FAE_MAX_TABLES + 1]; // prefix of sort tiles per table
    int32_t n_tables;
    int32_t dim;
    int32_t n_samples;
    int32_t shift, mask; // current radix digit
    int32_t *keys_in, *vals_in, *keys_out, *vals_out;
    int32_t *hist; // per table: [RADIX][tiles_z], concatenated
    int32_t *tot;  // [n_tables][RADIX]
    // single-kernel passes (chained tile prefixes)
    int32_t pass, n_passes, digit_bits, total_tiles;
    int32_t *ticket;   // [SWEEP_MAX_PASSES] next tile to hand out, per pass
    int32_t *ghist;    // [n_tables][SWEEP_MAX_PASSES][RADIX] digit counts of a table, per pass
    uint32_t *state;   // [SWEEP_MAX_PASSES][total_tiles][RADIX] flag (2 bits) | count (30 bits)
    // pooling / optimizer variants
    int32_t mean;      // every lookup receives its bag's gradient divided by the bag's length
    int32_t adagrad;   // row-wise Adagrad instead of plain SGD
    float eps;
    float *opt_state[FAE_MAX_TABLES]; // Adagrad: one accumulator per hot row
    const float *gout;
    int64_t gout_stride;
    float lr;
    float *partial;    // [total spans][2][dim]: sums of a span's first / last run when they cross its border
    int32_t *flags;    // [n_flags] one word per span: its border sums are published (zeroed by the sort stage)
    int32_t n_flags;
    int32_t fused_fixup; // border-crossing runs are finished inside the reduce kernel
    int32_t span;      // lookups per wave in the reduce kernel
    int32_t n_spans;   // total spans (blk_start then holds the span prefix per table)
    uint32_t *status;
    // debug outputs
    int32_t *dbg_uniq, *dbg_runlen, *dbg_table_start, *dbg_tile_sums, *dbg_rstart;
    int32_t dbg_tiles;
};

// ---------------------------------------------------------------------------------
// 1. keys
// ---------------------------------------------------------------------------------
#define KEYS_PER_THREAD 4
#define KEYS_PER_BLOCK (256 * KEYS_PER_THREAD)
#define SWEEP_MAX_PASSES 4
#define SWEEP_AGGREGATE 1u // the tile's own digit count is published
#define SWEEP_PREFIX 2u    // the count of this and all earlier tiles of the table is published
#define SWEEP_SPIN_LIMIT (1 << 22)

// Four consecutive lookups of one thread: (slot, sample) pairs, 16-byte loads and stores when
// aligned, plus the digit counts of every radix pass into the workgroup's LDS histograms.
__device__ __forceinline__ void bwd_keys_thread(const BwdArgs &a, int z, int j0, int n, const int32_t *off, int s_first,
                                                int (*s_hist)[RADIX])
{
    const int32_t *slots = a.slots[z] + j0;
    int32_t *ko = a.keys_in + a.seg_start[z] + j0;
    int32_t *vo = a.vals_in + a.seg_start[z] + j0;
    int k[KEYS_PER_THREAD], v[KEYS_PER_THREAD];
    const bool full = j0 + KEYS_PER_THREAD <= n;
    const bool aligned = full && ((((uintptr_t)slots) | ((uintptr_t)ko) | ((uintptr_t)vo)) & 15) == 0;
    if (aligned) {
        const int4 t = *(const int4 *)slots;
        k[0] = t.x; k[1] = t.y; k[2] = t.z; k[3] = t.w;
    } else {
#pragma unroll
        for (int q = 0; q < KEYS_PER_THREAD; ++q)
            k[q] = j0 + q < n ? slots[q] : 0;
    }
    bool bad = false;
    int s = off ? s_first : 0;
#pragma unroll
    for (int q = 0; q < KEYS_PER_THREAD; ++q) {
        const int j = j0 + q;
        if (j >= n)
            break;
        if ((unsigned)k[q] >= (unsigned)a.n_hot[z]) {
            bad = true;
            k[q] = a.n_hot[z]; // sorts behind every valid slot of the table; never dereferenced
        }
        if (off) {
            // bounded walk; a long stretch of empty bags falls back to a search
            int steps = 0;
            while (s + 1 < a.n_samples && off[s + 1] <= j) {
                ++s;
                if (++steps == 64) {
                    s = fae_sample_of(off, a.n_samples, j);
                    break;
                }
            }
            if (off[s] > j || off[s + 1] <= j)
                bad = true; // malformed CSR
            v[q] = s;
        } else {
            v[q] = j;
        }
    }
    if (bad)
        fae_flag(a.status, FAE_STATUS_ERANGE);
    if (a.n_passes > 0) { // digit counts of this table for every pass (their order does not matter)
#pragma unroll
        for (int q = 0; q < KEYS_PER_THREAD; ++q)
            if (j0 + q < n)
                for (int p = 0; p < a.n_passes; ++p)
                    atomicAdd(&s_hist[p][(k[q] >> (p * a.digit_bits)) & ((1 << a.digit_bits) - 1)], 1);
    }
    if (aligned) {
        *(int4 *)ko = make_int4(k[0], k[1], k[2], k[3]);
        *(int4 *)vo = make_int4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int q = 0; q < KEYS_PER_THREAD; ++q)
            if (j0 + q < n) {
                ko[q] = k[q];
                vo[q] = v[q];
            }
    }
}

// Every workgroup of a sort-stage kernel clears its slice of the span flags.  The slice length
// comes from the host (whole 256-byte pieces, so that two workgroups never share a cache line):
// reading the grid size on the device would put one more dependent scalar load in front of
// workgroups that live for a few microseconds.
__device__ __forceinline__ void bwd_clear_flags(int32_t *flags, int n_flags, int slice, int block_threads)
{
    const int beg = blockIdx.x * slice;
    const int end = beg + slice < n_flags ? beg + slice : n_flags;
    for (int i = beg + (int)threadIdx.x; i < end; i += block_threads)
        flags[i] = 0;
}
static inline int bwd_flag_slice(int64_t n_flags, int64_t blocks)
{
    const int64_t per = blocks > 0 ? (n_flags + blocks - 1) / blocks : n_flags;
    return (int)((per + 63) & ~(int64_t)63);
}

// Each thread handles four consecutive lookups (16-byte loads and stores when aligned).
__global__ __launch_bounds__(256) void bwd_keys_kernel(BwdArgs a)
{
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int j0 = (blockIdx.x - a.blk_start[z]) * KEYS_PER_BLOCK + threadIdx.x * KEYS_PER_THREAD;
    const int n = a.seg_start[z + 1] - a.seg_start[z];
    const int32_t *off = a.offsets[z];
    // sample of a lookup: one binary search per workgroup (its first lookup), then every thread
    // walks forward from there (a workgroup's lookups span few bags)
    __shared__ int s_first;
    __shared__ int s_hist[SWEEP_MAX_PASSES][RADIX];
    if (off && threadIdx.x == 0) {
        const int jb = (blockIdx.x - a.blk_start[z]) * KEYS_PER_BLOCK;
        s_first = fae_sample_of(off, a.n_samples, jb < n ? jb : n - 1);
    }
    for (int p = 0; p < a.n_passes; ++p)
        s_hist[p][threadIdx.x] = 0;
    __syncthreads();
    if (j0 < n)
        bwd_keys_thread(a, z, j0, n, off, s_first, s_hist);
    if (a.n_passes > 0) {
        __syncthreads();
        for (int p = 0; p < a.n_passes; ++p) {
            const int c = s_hist[p][threadIdx.x];
            if (c)
                atomicAdd(&a.ghist[(z * SWEEP_MAX_PASSES + p) * RADIX + threadIdx.x], c);
        }
    }
}

static_assert(sizeof(BwdArgs) <= 4096, "kernel arguments are passed by value");

// ---------------------------------------------------------------------------------
// 2. segmented LSD radix sort, one pass = histogram / column scan / scatter
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(SORT_THREADS) void sort_hist_kernel(BwdArgs a)
{
    __shared__ int cnt[RADIX];
    const int z = fae_find_table(a.tile_start, a.n_tables, blockIdx.x);
    const int tl = blockIdx.x - a.tile_start[z];
    const int tiles_z = a.tile_start[z + 1] - a.tile_start[z];
    const int seg1 = a.seg_start[z + 1];
    const int base = a.seg_start[z] + tl * SORT_TILE;
    cnt[threadIdx.x] = 0;
    __syncthreads();
    const int32_t *kp = a.keys_in + base;
    if (base + SORT_TILE <= seg1 && (((uintptr_t)kp) & 15) == 0) {
#pragma unroll
        for (int i = 0; i < SORT_ITEMS / 4; ++i) { // 16-byte loads; the count does not depend on the order
            const int4 t = ((const int4 *)kp)[i * SORT_THREADS + threadIdx.x];
            atomicAdd(&cnt[(t.x >> a.shift) & a.mask], 1);
            atomicAdd(&cnt[(t.y >> a.shift) & a.mask], 1);
            atomicAdd(&cnt[(t.z >> a.shift) & a.mask], 1);
            atomicAdd(&cnt[(t.w >> a.shift) & a.mask], 1);
        }
    } else {
#pragma unroll
        for (int i = 0; i < SORT_ITEMS; ++i) {
            int p = base + i * SORT_THREADS + threadIdx.x;
            if (p < seg1)
                atomicAdd(&cnt[(a.keys_in[p] >> a.shift) & a.mask], 1);
        }
    }
    __syncthreads();
    a.hist[RADIX * a.tile_start[z] + threadIdx.x * tiles_z + tl] = cnt[threadIdx.x];
}

// one wave per (table, digit): exclusive scan of that digit's counts over the table's tiles
__global__ __launch_bounds__(256) void sort_colscan_kernel(BwdArgs a)
{
    const int wid = blockIdx.x * (256 / FAE_WAVE) + threadIdx.x / FAE_WAVE;
    const int lane = fae_lane();
    if (wid >= a.n_tables * RADIX)
        return;
    const int z = wid / RADIX, d = wid % RADIX;
    const int tiles_z = a.tile_start[z + 1] - a.tile_start[z];
    int32_t *col = a.hist + RADIX * a.tile_start[z] + d * tiles_z;
    int carry = 0;
    for (int i0 = 0; i0 < tiles_z; i0 += FAE_WAVE) {
        int i = i0 + lane;
        int v = i < tiles_z ? col[i] : 0;
        int inc = fae_wave_incl_scan(v);
        if (i < tiles_z)
            col[i] = carry + inc - v;
        carry += __shfl(inc, FAE_WAVE - 1, FAE_WAVE);
    }
    if (lane == 0)
        a.tot[wid] = carry;
}

// Stable scatter of one tile.  Ranks come from a wave-level match on the digit plus per-wave
// counters; the tile is then put in digit order inside LDS so that the global writes of a
// digit are runs of consecutive addresses instead of single scattered words.
//
// ITEMS = keys per thread (a tile is 256 * ITEMS keys).
// CHAINED = false: the tile's output offsets come from the histogram / column-scan kernels.
// CHAINED = true : the whole pass is this one kernel.  Tiles are handed out in order by a
// ticket counter; a tile publishes its digit counts, then adds up the published counts of
// the tiles before it (walking back until it meets a tile that already published its
// running total) and publishes its own running total.  A tile only ever waits for tiles
// with smaller tickets, which are already running, so every wait ends; the wait is bounded
// anyway and reports an internal error instead of spinning forever.
template <bool CHAINED, int ITEMS> __global__ __launch_bounds__(SORT_THREADS) void sort_scatter_kernel(BwdArgs a)
{
    constexpr int TILE = SORT_THREADS * ITEMS;
    __shared__ int wcnt[SORT_WAVES][RADIX];  // per wave: running count, then start inside the tile
    __shared__ int gbase[RADIX];             // global position of the tile's first element of a digit
    __shared__ int tbase[RADIX];             // position inside the tile of the first element of a digit
    __shared__ int skey[TILE], sval[TILE];
    __shared__ int scan_lds[SORT_THREADS / FAE_WAVE + 1];
    __shared__ int s_tile;
    int tile = blockIdx.x;
    if (CHAINED) {
        if (threadIdx.x == 0)
            s_tile = atomicAdd(&a.ticket[a.pass], 1);
        __syncthreads();
        tile = s_tile;
    }
    const int z = fae_find_table(a.tile_start, a.n_tables, tile);
    const int tl = tile - a.tile_start[z];
    const int tiles_z = a.tile_start[z + 1] - a.tile_start[z];
    const int seg1 = a.seg_start[z + 1];
    const int w = threadIdx.x / FAE_WAVE, lane = fae_lane();
    const int tile0 = a.seg_start[z] + tl * TILE;
    const int base = tile0 + w * (FAE_WAVE * ITEMS);
    const int n_tile = seg1 - tile0 < TILE ? seg1 - tile0 : TILE;
    volatile int *my_cnt = wcnt[w];
#pragma unroll
    for (int i = 0; i < RADIX / FAE_WAVE; ++i)
        my_cnt[i * FAE_WAVE + lane] = 0;
    __builtin_amdgcn_wave_barrier();

    int key[ITEMS], val[ITEMS], off[ITEMS];
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int p = base + i * FAE_WAVE + lane;
        const bool valid = p < seg1;
        key[i] = valid ? a.keys_in[p] : 0;
        val[i] = valid ? a.vals_in[p] : 0;
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool valid = base + i * FAE_WAVE + lane < seg1;
        const int d = (key[i] >> a.shift) & a.mask;
        // lanes of this round that hold the same digit (valid lanes only)
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < RADIX_BITS; ++b) {
            const bool bit = (d >> b) & 1;
            const uint64_t m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        const int rank = __popcll(peers & lt_mask);
        const int n_peers = __popcll(peers);
        int old = 0;
        if (valid) {
            old = my_cnt[d];
            if (rank == 0)
                my_cnt[d] = old + n_peers;
        }
        __builtin_amdgcn_wave_barrier();
        off[i] = old + rank;
    }
    __syncthreads();
    {
        // thread t owns digit t: the four waves' counts -> starts inside the tile and in the output
        const int t = threadIdx.x;
        const int c0 = wcnt[0][t], c1 = wcnt[1][t], c2 = wcnt[2][t], c3 = wcnt[3][t];
        int total;
        if (!CHAINED) {
            const int ex = fae_block_excl_scan<SORT_THREADS>(a.tot[z * RADIX + t], scan_lds, &total);
            gbase[t] = a.seg_start[z] + ex + a.hist[RADIX * a.tile_start[z] + t * tiles_z + tl];
        } else {
            const uint32_t mine = (uint32_t)(c0 + c1 + c2 + c3);
            uint32_t *st = a.state + ((size_t)a.pass * a.total_tiles + tile) * RADIX + t;
            uint32_t before = 0; // lookups with digit t in the earlier tiles of this table
            if (tl == 0) {
                __hip_atomic_store(st, (SWEEP_PREFIX << 30) | mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                __hip_atomic_store(st, (SWEEP_AGGREGATE << 30) | mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                // Walk back over the earlier tiles of the table, eight at a time (their words are
                // loaded together; a tile that has published nothing yet is read again).  The
                // table's first tile publishes a running total, so the walk stops there at the latest.
                int back = 1; // distance of the nearest tile not yet added
                int spins = 0;
                bool done = false;
                while (!done) {
                    uint32_t v[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const int bq = back + q <= tl ? back + q : tl; // clamped into the table (tile tl back is its first)
                        v[q] = __hip_atomic_load(st - (size_t)bq * RADIX, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        if (done || back > tl)
                            break;
                        const uint32_t flag = v[q] >> 30;
                        if (flag == 0) { // not published yet: start the next round at this tile
                            if (++spins > SWEEP_SPIN_LIMIT) {
                                fae_flag(a.status, FAE_STATUS_EINTERNAL);
                                done = true;
                            } else {
                                __builtin_amdgcn_s_sleep(1);
                            }
                            break;
                        }
                        before += v[q] & 0x3fffffffu;
                        ++back;
                        if (flag == SWEEP_PREFIX)
                            done = true;
                    }
                    if (back > tl)
                        done = true; // cannot happen before a running total is met; keeps the walk inside the table
                }
                __hip_atomic_store(st, (SWEEP_PREFIX << 30) | (before + mine), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
            const int ex = fae_block_excl_scan<SORT_THREADS>(
                a.ghist[(z * SWEEP_MAX_PASSES + a.pass) * RADIX + t], scan_lds, &total);
            gbase[t] = a.seg_start[z] + ex + (int)before;
        }
        const int tb = fae_block_excl_scan<SORT_THREADS>(c0 + c1 + c2 + c3, scan_lds, &total);
        tbase[t] = tb;
        wcnt[0][t] = tb;
        wcnt[1][t] = tb + c0;
        wcnt[2][t] = tb + c0 + c1;
        wcnt[3][t] = tb + c0 + c1 + c2;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        if (base + i * FAE_WAVE + lane < seg1) {
            const int d = (key[i] >> a.shift) & a.mask;
            const int lp = wcnt[w][d] + off[i];
            skey[lp] = key[i];
            sval[lp] = val[i];
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int lp = i * SORT_THREADS + threadIdx.x;
        if (lp < n_tile) {
            const int k = skey[lp];
            const int d = (k >> a.shift) & a.mask;
            const int dst = gbase[d] + (lp - tbase[d]);
            a.keys_out[dst] = k;
            a.vals_out[dst] = sval[lp];
        }
    }
}

// ---------------------------------------------------------------------------------
// 2b. small tables: a table's list is sorted inside LDS by a few workgroups.
// Each workgroup loads all keys of its table (64 KiB of LDS, left in place), takes the
// keys whose top bits equal its part number (an ordered selection, so the input order
// survives), and LSD-sorts that subset on the remaining low bits.  What moves is a
// 16-bit permutation (position -> original lookup), ping-ponged between two 32 KiB
// arrays.  A radix pass makes two sweeps over the permutation: a per-wave digit
// histogram, then the same stable ranking as the global pass (wave-level match on
// the digit, running per-wave offsets).  The parts of a table are disjoint key ranges,
// so their outputs are laid end to end: part p starts after all keys of parts < p.
// ---------------------------------------------------------------------------------
struct LsortArgs {
    const int32_t *slots[FAE_MAX_TABLES];
    const int32_t *offsets[FAE_MAX_TABLES];
    int32_t n_hot[FAE_MAX_TABLES];
    int32_t seg_start[FAE_MAX_TABLES + 1];
    int32_t blk_start[FAE_MAX_TABLES + 1]; // workgroups per table (0 for tables sorted elsewhere)
    int32_t part_shift[FAE_MAX_TABLES];    // part of a key = key >> part_shift
    int32_t n_tables;
    int32_t n_samples;
    int32_t *keys_out, *vals_out;
    uint32_t *status;
    int32_t *flags; // span flags of the reduce kernel, zeroed here
    int32_t n_flags, flag_slice;
};

__global__ __launch_bounds__(LSORT_THREADS) void lds_sort_kernel(LsortArgs a)
{
    bwd_clear_flags(a.flags, a.n_flags, a.flag_slice, LSORT_THREADS);
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    lds_sort_block(a.slots[z], a.offsets[z], a.seg_start[z + 1] - a.seg_start[z], a.n_hot[z],
                   blockIdx.x - a.blk_start[z], a.part_shift[z], a.n_samples, a.keys_out + a.seg_start[z],
                   a.vals_out + a.seg_start[z], a.status);
}

// ---------------------------------------------------------------------------------
// 3 + 4. segment reduce + optimizer step
// ---------------------------------------------------------------------------------
template <typename V> struct bwd_vec;
template <> struct bwd_vec<float4> {
    static __device__ __forceinline__ float4 zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ __forceinline__ void add(float4 &a, const float4 &b)
    {
        a.x += b.x;
        a.y += b.y;
        a.z += b.z;
        a.w += b.w;
    }
    static __device__ __forceinline__ float4 sgd(const float4 &w, const float4 &g, float lr)
    {
        return make_float4(w.x - lr * g.x, w.y - lr * g.y, w.z - lr * g.z, w.w - lr * g.w);
    }
    static __device__ __forceinline__ void scale(float4 &a, float f)
    {
        a.x *= f;
        a.y *= f;
        a.z *= f;
        a.w *= f;
    }
    static __device__ __forceinline__ float sumsq(const float4 &a) { return (a.x * a.x + a.y * a.y) + (a.z * a.z + a.w * a.w); }
};
template <> struct bwd_vec<float> {
    static __device__ __forceinline__ float zero() { return 0.f; }
    static __device__ __forceinline__ void add(float &a, const float &b) { a += b; }
    static __device__ __forceinline__ float sgd(const float &w, const float &g, float lr) { return w - lr * g; }
    static __device__ __forceinline__ void scale(float &a, float f) { a *= f; }
    static __device__ __forceinline__ float sumsq(const float &a) { return a * a; }
};

template <typename V> __device__ __forceinline__ V bwd_shfl_up(const V &v, int d);
template <> __device__ __forceinline__ float4 bwd_shfl_up<float4>(const float4 &v, int d)
{
    return make_float4(__shfl_up(v.x, d, FAE_WAVE), __shfl_up(v.y, d, FAE_WAVE), __shfl_up(v.z, d, FAE_WAVE),
                       __shfl_up(v.w, d, FAE_WAVE));
}
template <> __device__ __forceinline__ float bwd_shfl_up<float>(const float &v, int d) { return __shfl_up(v, d, FAE_WAVE); }
template <typename V> __device__ __forceinline__ V bwd_shfl(const V &v, int src);
template <> __device__ __forceinline__ float4 bwd_shfl<float4>(const float4 &v, int src)
{
    return make_float4(__shfl(v.x, src, FAE_WAVE), __shfl(v.y, src, FAE_WAVE), __shfl(v.z, src, FAE_WAVE),
                       __shfl(v.w, src, FAE_WAVE));
}
template <> __device__ __forceinline__ float bwd_shfl<float>(const float &v, int src) { return __shfl(v, src, FAE_WAVE); }

// A slice of a border sum that another workgroup of the same launch reads: stored and loaded
// word by word with device-scope atomics, which go past the caches that are private to a part
// of the chip.  (Between two launches plain accesses are enough.)
__device__ __forceinline__ void bwd_store_shared(float4 *p, const float4 &v)
{
    float *f = (float *)p;
    __hip_atomic_store(f + 0, v.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(f + 1, v.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(f + 2, v.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(f + 3, v.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void bwd_store_shared(float *p, const float &v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float4 bwd_load_shared(const float4 *p)
{
    const float *f = (const float *)p;
    return make_float4(__hip_atomic_load(f + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                       __hip_atomic_load(f + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                       __hip_atomic_load(f + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                       __hip_atomic_load(f + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ float bwd_load_shared(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// What a span knows about its borders (same predicate in the reduce and the fix-up kernel).
struct SpanInfo {
    int z, seg0, seg1, pos0, pos1, first_key, last_key, local;
    bool head_open, tail_open;
};

__device__ __forceinline__ SpanInfo bwd_span_info(const BwdArgs &a, int sid)
{
    SpanInfo s;
    s.z = fae_find_table(a.blk_start, a.n_tables, sid);
    s.local = sid - a.blk_start[s.z];
    s.seg0 = a.seg_start[s.z];
    s.seg1 = a.seg_start[s.z + 1];
    s.pos0 = s.seg0 + s.local * a.span;
    s.pos1 = s.pos0 + a.span < s.seg1 ? s.pos0 + a.span : s.seg1;
    // four independent loads (indices clamped into the segment), no dependent branches
    s.first_key = a.keys_in[s.pos0];
    s.last_key = a.keys_in[s.pos1 - 1];
    const int before = a.keys_in[s.pos0 > s.seg0 ? s.pos0 - 1 : s.seg0];
    const int after = a.keys_in[s.pos1 < s.seg1 ? s.pos1 : s.seg1 - 1];
    s.head_open = s.pos0 > s.seg0 && before == s.first_key;
    s.tail_open = s.pos1 < s.seg1 && after == s.last_key;
    return s;
}

template <typename V, int LPR> __global__ __launch_bounds__(256) void bwd_reduce_kernel(BwdArgs a)
{
    constexpr int G = FAE_WAVE / LPR;              // lane groups = gradient rows per step
    constexpr int VW = sizeof(V) / sizeof(float);
    constexpr int STEPS = FAE_WAVE / G;            // steps per tile of 64 lookups
    constexpr int UN = STEPS < 4 ? STEPS : 4;      // steps whose loads are issued together
    const int sid = blockIdx.x * (256 / FAE_WAVE) + threadIdx.x / FAE_WAVE;
    if (sid >= a.n_spans)
        return;
    const SpanInfo sp = bwd_span_info(a, sid);
    const int lane = fae_lane(), g = lane / LPR, l = lane % LPR;
    const int ncols = a.dim / VW;
    const int n_hot = a.n_hot[sp.z];
    V *W = (V *)a.W[sp.z];
    const float *gbase = a.gout + (int64_t)sp.z * a.dim;
    V *part = (V *)(a.partial + (int64_t)sid * 2 * a.dim);

    for (int c0 = 0; c0 < ncols; c0 += LPR) {
        const int c = c0 + l;
        const bool active = c < ncols;
        // Sum of the run that is open at the end of the previous step.  It lives in the last lane
        // group only: the rotations of the scan below hand it to the groups that continue the run.
        V cv = bwd_vec<V>::zero();
        int klast = KEY_NONE; // last key of the previous tile (none at the span's start)
        int dist_in = 0;      // position inside its run of a lookup that continues the previous tile's last run
        for (int t0 = sp.pos0; t0 < sp.pos1; t0 += FAE_WAVE) {
            const int p = t0 + lane;
            const int kreg = p < sp.pos1 ? a.keys_in[p] : KEY_NONE;
            const int sreg = p < sp.pos1 ? a.vals_in[p] : 0;
            // key that follows each lookup; the span's last lookup always closes its run here
            int kafter = __shfl_down(kreg, 1, FAE_WAVE);
            if (lane == FAE_WAVE - 1)
                kafter = t0 + FAE_WAVE < sp.pos1 ? a.keys_in[t0 + FAE_WAVE] : KEY_NONE;
            if (p == sp.pos1 - 1)
                kafter = KEY_NONE;
            // where the finished run of lookup p goes: 0 nowhere (not the last of its run, or an
            // invalid slot), 1 SGD on its row, 2 / 3 the span's head / tail scratch row
            int dreg = 0;
            if (p < sp.pos1 && kafter != kreg && kreg < n_hot)
                dreg = (sp.head_open && kreg == sp.first_key) ? 2 : ((sp.tail_open && kreg == sp.last_key) ? 3 : 1);
            // dist = how many lookups of the same run precede lookup p inside this span (capped):
            // lookup p continues the sum of lookup p - d exactly when dist >= d, so the scan needs
            // no key comparisons across lanes.  From the run heads of the tile (one ballot).
            int kprev = __shfl_up(kreg, 1, FAE_WAVE);
            if (lane == 0)
                kprev = klast;
            const uint64_t heads = __ballot(kreg != kprev);
            const uint64_t upto = heads & (lane == FAE_WAVE - 1 ? ~0ull : ((2ull << lane) - 1ull));
            int dist = upto != 0 ? lane - (63 - __clzll(upto)) : lane + dist_in;
            dist = dist < 255 ? dist : 255;
            dreg |= dist << 2;
            float ireg = 1.0f; // mean pooling: 1 / (lookups in the lookup's bag)
            if (a.mean && a.offsets[sp.z] && p < sp.pos1) {
                const int32_t *off = a.offsets[sp.z];
                const int len = off[sreg + 1] - off[sreg];
                ireg = 1.0f / (float)(len > 0 ? len : 1);
            }
            klast = __builtin_amdgcn_readlane(kreg, FAE_WAVE - 1);
            dist_in = __builtin_amdgcn_readlane(dist, FAE_WAVE - 1) + 1;
            for (int i0 = 0; i0 < STEPS; i0 += UN) {
                if (t0 + i0 * G >= sp.pos1)
                    break;
                int kk[UN], dd[UN];
                V vv[UN], ww[UN];
                float inv[UN], sw[UN];
#pragma unroll
                for (int u = 0; u < UN; ++u) { // every load of the batch is issued before the first use
                    const int e = (i0 + u) * G + g;
                    kk[u] = __shfl(kreg, e, FAE_WAVE);
                    dd[u] = __shfl(dreg, e, FAE_WAVE);
                    const int s = __shfl(sreg, e, FAE_WAVE);
                    inv[u] = a.mean ? __shfl(ireg, e, FAE_WAVE) : 1.0f;
                    vv[u] = (active && kk[u] != KEY_NONE) ? ((const V *)(gbase + (int64_t)s * a.gout_stride))[c]
                                                         : bwd_vec<V>::zero();
                    ww[u] = (active && (dd[u] & 3) == 1) ? W[(int64_t)kk[u] * ncols + c] : bwd_vec<V>::zero();
                    sw[u] = (a.adagrad && (dd[u] & 3) == 1) ? a.opt_state[sp.z][kk[u]] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int kg = kk[u];
                    const int dest = dd[u] & 3, dist_u = dd[u] >> 2;
                    V vg = vv[u];
                    if (a.mean)
                        bwd_vec<V>::scale(vg, inv[u]);
                    // Inclusive segmented scan over the lane groups, the open run of the previous step
                    // standing in front of group 0: a rotation by d groups brings group g - d to
                    // group g, and the carried sum (held by the last group) to group d - 1.
#pragma unroll
                    for (int d = 1; d < G; d <<= 1) {
                        const V z = g == G - 1 ? cv : vg;
                        const V vp = bwd_shfl<V>(z, (lane - d * LPR) & (FAE_WAVE - 1));
                        if (dist_u >= d && g >= d - 1)
                            bwd_vec<V>::add(vg, vp);
                    }
                    if (g == G - 1 && dist_u >= G)
                        bwd_vec<V>::add(vg, cv); // the last group reaches back past group 0
                    float step = a.lr;
                    if (a.adagrad) { // one accumulator per row: grows by the row's mean squared gradient
                        float q = bwd_vec<V>::sumsq(vg);
#pragma unroll
                        for (int m = 1; m < LPR; m <<= 1)
                            q += __shfl_xor(q, m, FAE_WAVE);
                        const float acc = sw[u] + q / (float)a.dim;
                        step = a.lr / (sqrtf(acc) + a.eps);
                        if (dest == 1 && l == 0)
                            a.opt_state[sp.z][kg] = acc;
                    }
                    if (active) {
                        if (dest == 1)
                            W[(int64_t)kg * ncols + c] = bwd_vec<V>::sgd(ww[u], vg, step);
                        else if (dest == 2) {
                            if (a.fused_fixup)
                                bwd_store_shared(&part[c], vg);
                            else
                                part[c] = vg;
                        } else if (dest == 3) {
                            if (a.fused_fixup)
                                bwd_store_shared(&part[ncols + c], vg);
                            else
                                part[ncols + c] = vg;
                        }
                    }
                    cv = vg; // used from the last group only
                }
            }
        }
    }
    if (!a.fused_fixup)
        return;
    // Runs that cross span borders are finished here, by the span in which they end: it adds the
    // pieces the earlier spans have published (their tail sum where the run began, their whole-span
    // sums in between) to its own head sum and applies the update.  It only ever waits for spans
    // with smaller numbers, which were started before it; the wait is bounded all the same.
    const int c = l; // one column slice per lane: the host takes this path only when the row fits LPR lanes
    const bool active = c < ncols;
    if (sp.head_open || sp.tail_open) {
        __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0): this wave's border sums have been written
        if (lane == 0)
            __hip_atomic_store(&a.flags[sid], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const bool closes_head = sp.head_open && !(sp.first_key == sp.last_key && sp.tail_open);
    if (!closes_head || sp.first_key >= n_hot)
        return;
    const int k = sp.first_key;
    V *wp = W + (int64_t)k * ncols + c;
    V wv = bwd_vec<V>::zero();
    float sw = 0.f;
    if (g == 0 && active) {
        wv = *wp;
        if (a.adagrad)
            sw = a.opt_state[sp.z][k];
    }
    // earlier spans that lie wholly inside the run: the lookup before their first one has the key too
    int n_back = 0;
    for (int base = 0;; base += FAE_WAVE) {
        const int lm = sp.local - 1 - (base + lane);
        const bool inside = lm > 0 && a.keys_in[sp.seg0 + lm * a.span - 1] == k;
        const uint64_t m = __ballot(inside);
        const int cnt = m == ~0ull ? FAE_WAVE : __builtin_ctzll(~m);
        n_back += cnt;
        if (cnt < FAE_WAVE)
            break;
    }
    // pieces 0 .. n_back-1: whole-span sums of spans sid-1-t; piece n_back: tail sum of the span the run began in
    V acc = bwd_vec<V>::zero();
    constexpr int PB = 4; // pieces whose flags, then whose rows, are fetched together
    for (int t0 = g; t0 <= n_back; t0 += PB * G) {
        int spins = 0;
        for (;;) { // until the pieces of this round are all published
            int f[PB];
#pragma unroll
            for (int q = 0; q < PB; ++q) {
                const int t = t0 + q * G;
                f[q] = t <= n_back ? __hip_atomic_load(&a.flags[sid - 1 - t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 1;
            }
            bool all = true;
#pragma unroll
            for (int q = 0; q < PB; ++q)
                all = all && f[q] != 0;
            if (all)
                break;
            if (++spins > SWEEP_SPIN_LIMIT) {
                fae_flag(a.status, FAE_STATUS_EINTERNAL);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        V v[PB];
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int t = t0 + q * G;
            v[q] = bwd_vec<V>::zero();
            if (active && t <= n_back) {
                const V *row = (const V *)(a.partial + ((int64_t)(sid - 1 - t) * 2 + (t == n_back ? 1 : 0)) * a.dim);
                v[q] = bwd_load_shared(row + c);
            }
        }
#pragma unroll
        for (int q = 0; q < PB; ++q)
            bwd_vec<V>::add(acc, v[q]);
    }
#pragma unroll
    for (int mm = LPR; mm < FAE_WAVE; mm <<= 1) {
        const V o = bwd_shfl<V>(acc, lane ^ mm);
        bwd_vec<V>::add(acc, o);
    }
    if (g == 0 && active)
        bwd_vec<V>::add(acc, bwd_load_shared(part + c)); // this span's own piece of the run
    float step = a.lr;
    if (a.adagrad) {
        float q = active ? bwd_vec<V>::sumsq(acc) : 0.f;
#pragma unroll
        for (int mm = 1; mm < LPR; mm <<= 1)
            q += __shfl_xor(q, mm, FAE_WAVE);
        const float nacc = sw + q / (float)a.dim;
        step = a.lr / (sqrtf(nacc) + a.eps);
        if (g == 0 && l == 0)
            a.opt_state[sp.z][k] = nacc;
    }
    if (g == 0 && active)
        *wp = bwd_vec<V>::sgd(wv, acc, step);
}

// Segment reduce + SGD, second form: no traffic between lanes while the gradient rows are
// summed.  A wave still owns a span of sorted lookups, but each of its 64/LPR lane groups walks
// its own contiguous share of the span: NB gradient rows in flight per group and a running sum
// per run.  The (slot, sample) pairs are fetched one batch ahead (the same address in all lanes
// of a group), so the shape of the runs is known when a batch's loads are issued: the weight
// row of every run that closes strictly inside the share is loaded together with the gradient
// rows and updated as soon as the run's sum is complete.  What is left per group is its first
// and its last run; one pass over the groups, in order, joins those that continue each other
// and sends every joined run to its place: the weight row (preloaded by the group in which the
// run ends), or the span's head / tail scratch row when the run crosses the span's border (the
// fix-up kernel adds those up in span order, so the result does not depend on timing).
template <typename V, int LPR, int NB> __global__ __launch_bounds__(256) void bwd_reduce_walk_kernel(BwdArgs a)
{
    constexpr int G = FAE_WAVE / LPR;
    constexpr int VW = sizeof(V) / sizeof(float);
    const int sid = blockIdx.x * (256 / FAE_WAVE) + threadIdx.x / FAE_WAVE;
    if (sid >= a.n_spans)
        return;
    const SpanInfo sp = bwd_span_info(a, sid);
    const int lane = fae_lane(), g = lane / LPR, l = lane % LPR;
    const int ncols = a.dim / VW;
    const int n_hot = a.n_hot[sp.z];
    V *W = (V *)a.W[sp.z];
    const float *gbase = a.gout + (int64_t)sp.z * a.dim;
    V *part = (V *)(a.partial + (int64_t)sid * 2 * a.dim);
    const int share = a.span / G; // lookups per group (the span is a multiple of 64)
    const int q0 = sp.pos0 + g * share < sp.pos1 ? sp.pos0 + g * share : sp.pos1;
    const int q1 = q0 + share < sp.pos1 ? q0 + share : sp.pos1;

    for (int c0 = 0; c0 < ncols; c0 += LPR) {
        const int c = c0 + l;
        const bool active = c < ncols;
        // NB pairs of a batch and the key that follows them; KEY_NONE past the share's end
        auto load_pairs = [&](int j0, int *kk, int *ss) {
            if (NB % 4 == 0 && (j0 & 3) == 0 && j0 + NB <= q1) {
#pragma unroll
                for (int u = 0; u < NB; u += 4) {
                    const int4 k4 = *(const int4 *)(a.keys_in + j0 + u);
                    const int4 s4 = *(const int4 *)(a.vals_in + j0 + u);
                    kk[u] = k4.x; kk[u + 1] = k4.y; kk[u + 2] = k4.z; kk[u + 3] = k4.w;
                    ss[u] = s4.x; ss[u + 1] = s4.y; ss[u + 2] = s4.z; ss[u + 3] = s4.w;
                }
            } else {
#pragma unroll
                for (int u = 0; u < NB; ++u) {
                    kk[u] = j0 + u < q1 ? a.keys_in[j0 + u] : KEY_NONE;
                    ss[u] = j0 + u < q1 ? a.vals_in[j0 + u] : 0;
                }
            }
            kk[NB] = j0 + NB < q1 ? a.keys_in[j0 + NB] : KEY_NONE;
        };
        int cur = KEY_NONE;  // key of the run being summed
        V acc = bwd_vec<V>::zero();
        int hk = KEY_NONE;   // the share's first run, once it has closed inside the share
        V hv = bwd_vec<V>::zero();
        bool multi = false;  // a run has closed inside the share
        bool multi_ahead = false; // the same, as of the batch whose loads are being issued
        int kn[NB + 1], sn[NB];
        load_pairs(q0, kn, sn);
        for (int j0 = q0; j0 < q1; j0 += NB) {
            int kk[NB + 1], ss[NB];
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                kk[u] = kn[u];
                ss[u] = sn[u];
            }
            kk[NB] = kn[NB];
            V vv[NB], ww[NB];
            bool closes[NB];
            if (j0 + NB <= q1 && active) {
                // a full batch: every load is issued without a branch around it (a lookup that needs no
                // weight row reads row 0 of the table, a line that stays in the cache), and the
                // running sums are kept with selects instead of branches
#pragma unroll
                for (int u = 0; u < NB; ++u) {
                    vv[u] = ((const V *)(gbase + (int64_t)ss[u] * a.gout_stride))[c];
                    closes[u] = kk[u + 1] != KEY_NONE && kk[u + 1] != kk[u];
                    const bool need_w = closes[u] && multi_ahead && kk[u] < n_hot;
                    ww[u] = W[(int64_t)(need_w ? kk[u] : 0) * ncols + c];
                    multi_ahead = multi_ahead || closes[u];
                }
                load_pairs(j0 + NB, kn, sn);
#pragma unroll
                for (int u = 0; u < NB; ++u) {
                    const bool same = kk[u] == cur;
                    V t = vv[u];
                    if (same)
                        bwd_vec<V>::add(t, acc);
                    acc = t;
                    cur = kk[u];
                    const bool first_close = closes[u] && !multi;
                    if (first_close) {
                        hk = cur;
                        hv = acc;
                    }
                    if (closes[u] && multi && cur < n_hot)
                        W[(int64_t)cur * ncols + c] = bwd_vec<V>::sgd(ww[u], acc, a.lr);
                    multi = multi || closes[u];
                }
                continue;
            }
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                vv[u] = (active && kk[u] != KEY_NONE) ? ((const V *)(gbase + (int64_t)ss[u] * a.gout_stride))[c]
                                                     : bwd_vec<V>::zero();
                // a run closes here if another key follows inside the share
                closes[u] = kk[u] != KEY_NONE && kk[u + 1] != KEY_NONE && kk[u + 1] != kk[u];
                const bool need_w = closes[u] && multi_ahead && active && kk[u] < n_hot;
                ww[u] = need_w ? W[(int64_t)kk[u] * ncols + c] : bwd_vec<V>::zero();
                multi_ahead = multi_ahead || closes[u];
            }
            load_pairs(j0 + NB, kn, sn); // past the share's end it loads nothing
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int k = kk[u];
                if (k == KEY_NONE)
                    continue;
                if (k == cur) {
                    bwd_vec<V>::add(acc, vv[u]);
                } else {
                    cur = k;
                    acc = vv[u];
                }
                if (closes[u]) {
                    if (!multi) {
                        hk = cur;
                        hv = acc;
                        multi = true;
                    } else if (active && cur < n_hot) {
                        W[(int64_t)cur * ncols + c] = bwd_vec<V>::sgd(ww[u], acc, a.lr);
                    }
                }
            }
        }
        // weight rows of the group's first and last run, for whichever joined run ends there
        const V wh = (multi && active && hk < n_hot) ? W[(int64_t)hk * ncols + c] : bwd_vec<V>::zero();
        const V wt = (cur != KEY_NONE && active && cur < n_hot) ? W[(int64_t)cur * ncols + c] : bwd_vec<V>::zero();
        // a joined run with key k and sum v that ends in group `at` (as its first run if head)
        auto flush = [&](int at, bool head, int k, const V &v) {
            if (g != at || !active || k >= n_hot)
                return;
            if (sp.head_open && k == sp.first_key)
                part[c] = v;
            else if (sp.tail_open && k == sp.last_key)
                part[ncols + c] = v;
            else
                W[(int64_t)k * ncols + c] = bwd_vec<V>::sgd(head ? wh : wt, v, a.lr);
        };
        int ck = KEY_NONE, gprev = 0;
        V cv = bwd_vec<V>::zero();
#pragma unroll
        for (int gp = 0; gp < G; ++gp) {
            const int e_tk = __builtin_amdgcn_readlane(cur, gp * LPR);
            if (e_tk == KEY_NONE)
                continue; // an empty share (only past the span's end)
            const int e_multi = __builtin_amdgcn_readlane((int)multi, gp * LPR);
            const int e_hk = __builtin_amdgcn_readlane(hk, gp * LPR);
            const V e_tv = bwd_shfl<V>(acc, gp * LPR + l);
            const V e_hv = bwd_shfl<V>(hv, gp * LPR + l);
            const int fk = e_multi ? e_hk : e_tk; // key of the share's first run
            V first = e_multi ? e_hv : e_tv;
            if (fk == ck)
                bwd_vec<V>::add(first, cv); // continues the run carried over from the shares before
            else if (ck != KEY_NONE)
                flush(gprev, false, ck, cv);
            if (e_multi) {
                flush(gp, true, fk, first);
                ck = e_tk;
                cv = e_tv;
            } else {
                ck = fk;
                cv = first;
            }
            gprev = gp;
        }
        if (ck != KEY_NONE)
            flush(gprev, false, ck, cv);
    }
}

// one wave per span: if a run starts in this span and continues past its end, add the
// pieces (this span's tail, the following spans' heads) and apply the update.  The lanes
// find the extent of the run together (64 following spans per ballot) and the lane groups
// add alternate heads; the order of the additions is fixed by the span numbers.
template <typename V, int LPR> __global__ __launch_bounds__(256) void bwd_fixup_kernel(BwdArgs a)
{
    constexpr int G = FAE_WAVE / LPR;
    constexpr int VW = sizeof(V) / sizeof(float);
    const int sid = blockIdx.x * (256 / FAE_WAVE) + threadIdx.x / FAE_WAVE;
    if (sid >= a.n_spans)
        return;
    const int lane = fae_lane(), g = lane / LPR, l = lane % LPR;
    // Two dependent rounds of memory traffic only: (1) the span's border keys together with the
    // first keys of the next 64 spans, (2) the partial sums together with the weight row.
    const SpanInfo sp = bwd_span_info(a, sid);
    const int spans_z = a.blk_start[sp.z + 1] - a.blk_start[sp.z];
    const int j0 = sp.local + 1 + lane;
    const int follow_key = j0 < spans_z ? a.keys_in[sp.seg0 + j0 * a.span] : KEY_NONE;
    if (!sp.tail_open || (sp.head_open && sp.first_key == sp.last_key))
        return; // nothing crosses the end, or the run began in an earlier span
    const int k = sp.last_key;
    if (k >= a.n_hot[sp.z])
        return;
    // following spans that begin with the same key continue the run (keys are sorted)
    uint64_t m = __ballot(follow_key == k);
    int n_follow = m == ~0ull ? FAE_WAVE : __builtin_ctzll(~m);
    for (int base = sp.local + 1 + FAE_WAVE; n_follow == base - sp.local - 1 && base < spans_z; base += FAE_WAVE) {
        const int j = base + lane;
        const bool same = j < spans_z && a.keys_in[sp.seg0 + j * a.span] == k;
        m = __ballot(same);
        n_follow += m == ~0ull ? FAE_WAVE : __builtin_ctzll(~m);
    }
    const int ncols = a.dim / VW;
    const int first_sid = sid - sp.local;
    for (int c0 = 0; c0 < ncols; c0 += LPR) {
        const int c = c0 + l;
        V acc = bwd_vec<V>::zero();
        V tail = bwd_vec<V>::zero(), wv = bwd_vec<V>::zero();
        V *wp = (V *)a.W[sp.z] + (int64_t)k * ncols + c;
        if (c < ncols) {
            if (g == 0) { // issued together with the heads below
                tail = ((const V *)(a.partial + ((int64_t)sid * 2 + 1) * a.dim))[c];
                wv = *wp;
            }
            for (int j = g; j < n_follow; j += G)
                bwd_vec<V>::add(acc, ((const V *)(a.partial + (int64_t)(first_sid + sp.local + 1 + j) * 2 * a.dim))[c]);
        }
#pragma unroll
        for (int mm = LPR; mm < FAE_WAVE; mm <<= 1) {
            const V o = bwd_shfl<V>(acc, lane ^ mm);
            bwd_vec<V>::add(acc, o);
        }
        if (g == 0 && c < ncols)
            bwd_vec<V>::add(acc, tail);
        float step = a.lr;
        if (a.adagrad) { // group 0 holds the row's whole gradient; lanes past the row hold zeros
            float q = c < ncols ? bwd_vec<V>::sumsq(acc) : 0.f;
#pragma unroll
            for (int mm = 1; mm < LPR; mm <<= 1)
                q += __shfl_xor(q, mm, FAE_WAVE);
            if (g == 0) {
                const float nacc = a.opt_state[sp.z][k] + q / (float)a.dim;
                step = a.lr / (sqrtf(nacc) + a.eps);
                if (l == 0)
                    a.opt_state[sp.z][k] = nacc;
            }
        }
        if (g == 0 && c < ncols)
            *wp = bwd_vec<V>::sgd(wv, acc, step);
    }
}

// ---------------------------------------------------------------------------------
// debug outputs: distinct slots per table (ascending) and their multiplicities
// ---------------------------------------------------------------------------------
__device__ __forceinline__ bool dbg_is_head(const BwdArgs &a, int p)
{
    int z = 0;
    while (z + 1 < a.n_tables && p >= a.seg_start[z + 1])
        ++z;
    return p == a.seg_start[z] || a.keys_in[p] != a.keys_in[p - 1];
}

__global__ __launch_bounds__(256) void dbg_count_kernel(BwdArgs a)
{
    __shared__ int lds[256 / FAE_WAVE + 1];
    const int n = a.seg_start[a.n_tables];
    int c = 0;
    for (int k = 0; k < DBG_TILE / 256; ++k) {
        int p = blockIdx.x * DBG_TILE + threadIdx.x * (DBG_TILE / 256) + k;
        if (p < n && dbg_is_head(a, p))
            ++c;
    }
    int total;
    (void)fae_block_excl_scan<256>(c, lds, &total);
    if (threadIdx.x == 0)
        a.dbg_tile_sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void dbg_emit_kernel(BwdArgs a)
{
    __shared__ int lds[256 / FAE_WAVE + 1];
    const int n = a.seg_start[a.n_tables];
    bool head[DBG_TILE / 256];
    int c = 0;
    for (int k = 0; k < DBG_TILE / 256; ++k) {
        int p = blockIdx.x * DBG_TILE + threadIdx.x * (DBG_TILE / 256) + k;
        head[k] = p < n && dbg_is_head(a, p);
        c += head[k] ? 1 : 0;
    }
    int total;
    int ex = fae_block_excl_scan<256>(c, lds, &total);
    int u = a.dbg_tile_sums[blockIdx.x] + ex;
    for (int k = 0; k < DBG_TILE / 256; ++k) {
        int p = blockIdx.x * DBG_TILE + threadIdx.x * (DBG_TILE / 256) + k;
        if (p < n) {
            for (int z = 0; z < a.n_tables; ++z)
                if (a.seg_start[z] == p)
                    a.dbg_table_start[z] = u; // heads before p; also right for empty tables at p
            if (head[k]) {
                a.dbg_uniq[u] = a.keys_in[p];
                a.dbg_rstart[u] = p;
                ++u;
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const int U = a.dbg_tile_sums[a.dbg_tiles];
        for (int z = 0; z <= a.n_tables; ++z)
            if (a.seg_start[z] == n)
                a.dbg_table_start[z] = U;
        a.dbg_rstart[U] = n;
    }
}

__global__ __launch_bounds__(256) void dbg_runlen_kernel(BwdArgs a)
{
    const int U = a.dbg_tile_sums[a.dbg_tiles];
    for (int u = blockIdx.x * 256 + threadIdx.x; u < U; u += gridDim.x * 256)
        a.dbg_runlen[u] = a.dbg_rstart[u + 1] - a.dbg_rstart[u];
}

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------
namespace {
struct BwdPlan {
    int64_t N;
    int64_t tiles;
    int64_t small_tiles; // tiles of SORT_TILE_SMALL keys
    int64_t max_spans; // with the smallest span
    int64_t dbg_tiles;
};

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

struct BwdWs {
    int32_t *keys[2], *vals[2];
    int32_t *hist, *tot;
    uint32_t *sweep; // ticket[64] | ghist[nt][SWEEP_MAX_PASSES][RADIX] | state[SWEEP_MAX_PASSES][tiles][RADIX]
    float *partial;
    int32_t *flags;
    int64_t n_flags;
    int32_t *dbg_tile_sums, *dbg_rstart;
    bool ok;
    size_t used;
};

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

template <typename V, int LPR> void launch_reduce(fae_ctx *ctx, const BwdArgs &a)
{
    {
        fae_ktimer kt(ctx, FAE_K_BWD_REDUCE);
        const dim3 grid((a.n_spans + 3) / 4);
        if (ctx->opt_reduce != 2 || a.mean || a.adagrad) // the variants exist in the scan form only
            hipLaunchKernelGGL((bwd_reduce_kernel<V, LPR>), grid, dim3(256), 0, ctx->stream, a);
        else if (ctx->opt_unroll == 8)
            hipLaunchKernelGGL((bwd_reduce_walk_kernel<V, LPR, 8>), grid, dim3(256), 0, ctx->stream, a);
        else
            hipLaunchKernelGGL((bwd_reduce_walk_kernel<V, LPR, 4>), grid, dim3(256), 0, ctx->stream, a);
    }
    if (a.fused_fixup)
        return;
    fae_ktimer kt(ctx, FAE_K_BWD_FIXUP);
    hipLaunchKernelGGL((bwd_fixup_kernel<V, LPR>), dim3((a.n_spans + 3) / 4), dim3(256), 0, ctx->stream, a);
}

#define BWD_LPR_SWITCH(V, lpr, CALL)      \
    switch (lpr) {                        \
    case 1: CALL(V, 1); break;            \
    case 2: CALL(V, 2); break;            \
    case 4: CALL(V, 4); break;            \
    case 8: CALL(V, 8); break;            \
    case 16: CALL(V, 16); break;          \
    case 32: CALL(V, 32); break;          \
    default: CALL(V, 64); break;          \
    }
} // namespace

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

namespace {
// Common set-up of the backward: validation, workspace carving, per-table descriptors.
struct BwdSetup {
    BwdPlan plan;
    BwdWs w;
    BwdArgs a;
    bool empty;
};

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

// Workgroups per small table for the LDS sort: enough parts to occupy the chip, never lists
// below ~512 lookups.  part_shift[z]: part of a key = key >> shift; blk_start: prefix of
// workgroups per table (tables not sorted in LDS get none).  Returns the number of workgroups.
int lsort_plan(const fae_ctx *ctx, const fae_tables *hot_tables, const fae_batch *hot_batch, const bool *in_lds,
               int n_lds, int32_t *blk_start, int32_t *part_shift)
{
    const int nt = hot_tables->n_tables;
    int want = 1;
    while (want < 16 && n_lds * want * 2 <= ctx->n_cu)
        want <<= 1;
    int nb = 0;
    for (int z = 0; z < nt; ++z) {
        blk_start[z] = nb;
        if (!in_lds[z])
            continue;
        int kbits = 1; // bits of the largest key (n_hot itself marks an invalid slot)
        while ((hot_tables->h_rows[z] >> kbits) != 0)
            ++kbits;
        int parts = want;
        while (parts > 1 && hot_batch->h_n_lookups[z] / parts < 512)
            parts >>= 1;
        int pbits = 0;
        while ((1 << pbits) < parts)
            ++pbits;
        if (pbits > kbits)
            pbits = kbits;
        part_shift[z] = kbits - pbits;
        nb += (int)(hot_tables->h_rows[z] >> part_shift[z]) + 1; // parts that can hold a key: 0 .. (n_hot >> shift)
    }
    blk_start[nt] = nb;
    return nb;
}

// Steps 1 + 2 on stream `st`: (slot, sample) pairs sorted by slot per table.  *cur_out names
// the ping-pong buffer that holds the result.
int32_t bwd_sort_stage(fae_ctx *ctx, hipStream_t st, const fae_tables *hot_tables, const fae_batch *hot_batch,
                       BwdSetup &su, int *cur_out)
{
    BwdArgs &a = su.a;
    const BwdWs &w = su.w;
    const int nt = hot_tables->n_tables;
    // Tables whose lookups fit one workgroup are sorted in LDS; they take no part in the
    // global passes (zero tiles, zero key blocks).
    bool in_lds[FAE_MAX_TABLES];
    int n_lds = 0;
    int64_t max_hot_global = 0;
    int64_t tiles = 0;
    for (int z = 0; z < nt; ++z) {
        const int64_t nl = hot_batch->h_n_lookups[z];
        in_lds[z] = ctx->opt_sort != 1 && nl > 0 && nl <= LSORT_MAX;
        if (in_lds[z])
            ++n_lds;
        else if (nl > 0 && hot_tables->h_rows[z] > max_hot_global)
            max_hot_global = hot_tables->h_rows[z];
        a.tile_start[z] = (int32_t)tiles;
        if (!in_lds[z])
            tiles += (nl + SORT_TILE - 1) / SORT_TILE;
    }
    a.tile_start[nt] = (int32_t)tiles;
    // only the bits a slot (or the invalid marker n_hot) can occupy are sorted
    int bits = 1;
    while ((max_hot_global >> bits) != 0)
        ++bits;
    const int passes = tiles > 0 ? (bits + RADIX_BITS - 1) / RADIX_BITS : 0;
    const int digit_bits = passes > 0 ? (bits + passes - 1) / passes : RADIX_BITS;
    // Short lists: one kernel per pass (tiles chained through published counts), which saves
    // two launches per pass where launches are what a pass costs.  Long lists keep the
    // three-kernel passes: there the chained kernel's waits cost as much as the launches
    // (measured: 59 us against 63 us per pass at 10.5 M lookups, 16 us against 30 us at 0.2 M).
    // The chained kernel's counters start at zero; the keys kernel fills the per-table digit
    // histograms of all passes.  sort_variant 1 forces the three-kernel passes, 3 the chained ones.
    const bool chained = passes > 0 && ctx->opt_sort != 1 && (ctx->opt_sort == 3 || tiles <= 4LL * ctx->n_cu);
    // A chained pass over a short list takes small tiles: more workgroups, a shorter chain per tile
    // (the same rule sizes the workspace, so it goes by the lookups of all tables).
    const bool small_tiles = chained && su.plan.small_tiles <= SORT_SMALL_MAX_TILES;
    if (small_tiles) {
        tiles = 0;
        for (int z = 0; z < nt; ++z) {
            a.tile_start[z] = (int32_t)tiles;
            if (!in_lds[z])
                tiles += (hot_batch->h_n_lookups[z] + SORT_TILE_SMALL - 1) / SORT_TILE_SMALL;
        }
        a.tile_start[nt] = (int32_t)tiles;
    }
    if (chained) {
        a.n_passes = passes;
        a.digit_bits = digit_bits;
        a.total_tiles = (int32_t)tiles;
        a.ticket = (int32_t *)w.sweep;
        a.ghist = (int32_t *)w.sweep + 64;
        a.state = w.sweep + 64 + (size_t)nt * SWEEP_MAX_PASSES * RADIX;
    }
    if (tiles > 0) {
        // The span flags of the reduce kernel start at zero too.  The LDS sort clears them itself;
        // a batch with tables on the global passes gets them cleared here, together with the
        // chained passes' counters that follow them in the workspace.  (Clearing them in the keys
        // kernel instead cost that kernel a third of its time.)
        int64_t words = a.n_flags;
        if (chained)
            words = ((int32_t *)w.sweep - w.flags) +
                    (64 + ((int64_t)nt * SWEEP_MAX_PASSES + (int64_t)passes * tiles) * RADIX);
        int32_t rc = fae_fill_u32_on(ctx, st, w.flags, words, 0u);
        if (rc != FAE_OK)
            return rc;
    }
    // 1. keys
    {
        int64_t blocks = 0;
        for (int z = 0; z < nt; ++z) {
            a.blk_start[z] = (int32_t)blocks;
            if (!in_lds[z])
                blocks += (hot_batch->h_n_lookups[z] + KEYS_PER_BLOCK - 1) / KEYS_PER_BLOCK;
        }
        a.blk_start[nt] = (int32_t)blocks;
        a.keys_in = w.keys[0];
        a.vals_in = w.vals[0];
        if (blocks > 0) {
            fae_ktimer kt(ctx, FAE_K_BWD_KEYS, st);
            hipLaunchKernelGGL(bwd_keys_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a);
            FAE_LAUNCH_CHECK(ctx);
        }
    }
    // 2. sort
    int cur = 0;
    for (int pass = 0; pass < passes; ++pass) {
        a.pass = pass;
        a.shift = pass * digit_bits;
        a.mask = (1 << digit_bits) - 1;
        a.keys_in = w.keys[cur];
        a.vals_in = w.vals[cur];
        a.keys_out = w.keys[cur ^ 1];
        a.vals_out = w.vals[cur ^ 1];
        if (chained) {
            fae_ktimer kt(ctx, FAE_K_SORT_SCATTER, st);
            if (small_tiles)
                hipLaunchKernelGGL((sort_scatter_kernel<true, SORT_ITEMS_SMALL>), dim3((unsigned)tiles), dim3(SORT_THREADS), 0, st, a);
            else
                hipLaunchKernelGGL((sort_scatter_kernel<true, SORT_ITEMS>), dim3((unsigned)tiles), dim3(SORT_THREADS), 0, st, a);
            FAE_LAUNCH_CHECK(ctx);
            cur ^= 1;
            continue;
        }
        {
            fae_ktimer kt(ctx, FAE_K_SORT_HIST, st);
            hipLaunchKernelGGL(sort_hist_kernel, dim3((unsigned)tiles), dim3(SORT_THREADS), 0, st, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        {
            fae_ktimer kt(ctx, FAE_K_SORT_COLSCAN, st);
            hipLaunchKernelGGL(sort_colscan_kernel, dim3((unsigned)((nt * RADIX + 3) / 4)), dim3(256), 0, st, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        {
            fae_ktimer kt(ctx, FAE_K_SORT_SCATTER, st);
            hipLaunchKernelGGL((sort_scatter_kernel<false, SORT_ITEMS>), dim3((unsigned)tiles), dim3(SORT_THREADS), 0, st, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        cur ^= 1;
    }
    a.keys_in = w.keys[cur];
    a.vals_in = w.vals[cur];
    a.keys_out = nullptr;
    a.vals_out = nullptr;
    if (n_lds > 0) { // small tables: straight from the slots into the final buffer
        LsortArgs la;
        memset(&la, 0, sizeof(la));
        for (int z = 0; z < nt; ++z) {
            la.slots[z] = a.slots[z];
            la.offsets[z] = a.offsets[z];
            la.n_hot[z] = a.n_hot[z];
            la.seg_start[z] = a.seg_start[z];
        }
        const int nb = lsort_plan(ctx, hot_tables, hot_batch, in_lds, n_lds, la.blk_start, la.part_shift);
        la.seg_start[nt] = a.seg_start[nt];
        la.n_tables = nt;
        la.n_samples = a.n_samples;
        la.keys_out = w.keys[cur];
        la.vals_out = w.vals[cur];
        la.status = ctx->d_block;
        la.flags = a.flags;
        la.n_flags = a.n_flags;
        la.flag_slice = bwd_flag_slice(a.n_flags, nb);
        fae_ktimer kt(ctx, FAE_K_LDS_SORT, st);
        hipLaunchKernelGGL(lds_sort_kernel, dim3(nb), dim3(LSORT_THREADS), 0, st, la);
        FAE_LAUNCH_CHECK(ctx);
    }
    *cur_out = cur;
    return FAE_OK;
}
} // namespace

extern "C" int32_t fae_embbag_bwd_presort(fae_ctx *ctx, const fae_tables *hot_tables, const fae_batch *hot_batch,
                                          void *ws, size_t ws_bytes)
{
    BwdSetup su;
    int32_t rc = bwd_setup(ctx, hot_tables, hot_batch, ws, ws_bytes, "fae_embbag_bwd_presort", &su);
    if (rc != FAE_OK)
        return rc;
    ctx->presort.valid = false;
    if (su.empty)
        return FAE_OK;
    FAE_HIP(ctx, hipSetDevice(ctx->device));
    // fork: the side stream starts after everything already queued on the main stream
    // (earlier users of this workspace, producers of the slots)
    FAE_HIP(ctx, hipEventRecord(ctx->ev_fork, ctx->stream));
    FAE_HIP(ctx, hipStreamWaitEvent(ctx->aux_stream, ctx->ev_fork, 0));
    int cur = 0;
    rc = bwd_sort_stage(ctx, ctx->aux_stream, hot_tables, hot_batch, su, &cur);
    if (rc != FAE_OK)
        return rc;
    FAE_HIP(ctx, hipEventRecord(ctx->ev_join, ctx->aux_stream));
    ctx->presort.valid = true;
    ctx->presort.side = true;
    ctx->presort.ws = ws;
    ctx->presort.first_indices = hot_batch->h_indices[0];
    ctx->presort.n_samples = hot_batch->n_samples;
    ctx->presort.n_lookups = su.plan.N;
    ctx->presort.cur = cur;
    return FAE_OK;
}

// ---------------------------------------------------------------------------------
// Forward and the backward's sort in one launch (one-hot tables whose lists fit the LDS
// sort): the first workgroups sort, the rest copy rows.  The two roles share nothing but
// the slot lists they both read; the sort is latency/ALU bound on a few CUs while the
// row copies stream through the others, so the pair takes about as long as the slower one.
// ---------------------------------------------------------------------------------
struct FusedArgs {
    const float *W[FAE_MAX_TABLES];
    const int32_t *slots[FAE_MAX_TABLES];
    int32_t n_hot[FAE_MAX_TABLES];
    int32_t seg_start[FAE_MAX_TABLES + 1];
    int32_t sort_blk_start[FAE_MAX_TABLES + 1];
    int32_t part_shift[FAE_MAX_TABLES];
    int32_t n_tables, dim, n_samples;
    int32_t n_sort_blocks, fwd_blocks_per_table;
    int64_t out_stride;
    float *out;
    int32_t *keys_out, *vals_out;
    uint32_t *status;
    int32_t stream_out;
    int32_t *flags; // span flags of the reduce kernel, zeroed here
    int32_t n_flags, flag_slice;
};

template <typename V, int LPR> __global__ __launch_bounds__(LSORT_THREADS) void fwd_sort_kernel(FusedArgs a)
{
    bwd_clear_flags(a.flags, a.n_flags, a.flag_slice, LSORT_THREADS);
    if ((int)blockIdx.x < a.n_sort_blocks) {
        const int z = fae_find_table(a.sort_blk_start, a.n_tables, blockIdx.x);
        lds_sort_block(a.slots[z], nullptr, a.seg_start[z + 1] - a.seg_start[z], a.n_hot[z],
                       blockIdx.x - a.sort_blk_start[z], a.part_shift[z], a.n_samples, a.keys_out + a.seg_start[z],
                       a.vals_out + a.seg_start[z], a.status);
    } else {
        const int b = blockIdx.x - a.n_sort_blocks;
        const int z = b / a.fwd_blocks_per_table, bl = b % a.fwd_blocks_per_table;
        const int64_t s0 = ((int64_t)bl * LSORT_WAVES + threadIdx.x / FAE_WAVE) * FAE_WAVE;
        fwd_onehot_wave<V, LPR>((const V *)a.W[z], a.slots[z], a.n_hot[z], s0, a.n_samples, a.out + (int64_t)z * a.dim,
                                a.out_stride, a.dim, a.status, a.stream_out != 0);
    }
}

template <int LPR> static void launch_fwd_sort(fae_ctx *ctx, const FusedArgs &a, int blocks)
{
    hipLaunchKernelGGL((fwd_sort_kernel<float4, LPR>), dim3(blocks), dim3(LSORT_THREADS), 0, ctx->stream, a);
}

extern "C" int32_t fae_embbag_fwd_presort(fae_ctx *ctx, const fae_tables *hot_tables, const float *const *h_hotW,
                                          const fae_batch *hot_batch, float *out, int64_t out_row_stride, void *ws,
                                          size_t ws_bytes)
{
    BwdSetup su;
    int32_t rc = bwd_setup(ctx, hot_tables, hot_batch, ws, ws_bytes, "fae_embbag_fwd_presort", &su);
    if (rc != FAE_OK)
        return rc;
    const int nt = hot_tables->n_tables, dim = hot_tables->dim;
    const int64_t S = hot_batch->n_samples;
    // the fused launch covers the common case of the paper's workloads (every table one-hot,
    // batch within the LDS sort's reach, 16-byte aligned rows); anything else: plain forward
    bool fused = !su.empty && ctx->opt_sort != 1 && ctx->opt_fwd == 0 && h_hotW && out && dim % 4 == 0 &&
                 out_row_stride % 4 == 0 && out_row_stride >= (int64_t)nt * dim && ((uintptr_t)out) % 16 == 0 &&
                 S <= LSORT_MAX;
    for (int z = 0; fused && z < nt; ++z)
        fused = su.a.offsets[z] == nullptr && h_hotW[z] && ((uintptr_t)h_hotW[z]) % 16 == 0;
    if (!fused)
        return fae_embbag_fwd(ctx, hot_tables, h_hotW, hot_batch, out, out_row_stride);
    FAE_HIP(ctx, hipSetDevice(ctx->device));
    FusedArgs f;
    memset(&f, 0, sizeof(f));
    bool in_lds[FAE_MAX_TABLES];
    for (int z = 0; z < nt; ++z) {
        f.W[z] = h_hotW[z];
        f.slots[z] = su.a.slots[z];
        f.n_hot[z] = su.a.n_hot[z];
        f.seg_start[z] = su.a.seg_start[z];
        in_lds[z] = true;
    }
    f.seg_start[nt] = su.a.seg_start[nt];
    f.n_sort_blocks = lsort_plan(ctx, hot_tables, hot_batch, in_lds, nt, f.sort_blk_start, f.part_shift);
    f.n_tables = nt;
    f.dim = dim;
    f.n_samples = (int32_t)S;
    f.fwd_blocks_per_table = (int32_t)((S + LSORT_THREADS - 1) / LSORT_THREADS);
    f.out_stride = out_row_stride;
    f.out = out;
    f.keys_out = su.w.keys[0];
    f.vals_out = su.w.vals[0];
    f.status = ctx->d_block;
    f.stream_out = ctx->opt_fwd_stream != 0;
    f.flags = su.a.flags;
    f.n_flags = su.a.n_flags;
    const int blocks = f.n_sort_blocks + f.fwd_blocks_per_table * nt;
    f.flag_slice = bwd_flag_slice(f.n_flags, blocks);
    int lpr = 1;
    while (lpr < dim / 4 && lpr < 64)
        lpr <<= 1;
    {
        fae_ktimer kt(ctx, FAE_K_FWD_SORT);
        switch (lpr) {
        case 1: launch_fwd_sort<1>(ctx, f, blocks); break;
        case 2: launch_fwd_sort<2>(ctx, f, blocks); break;
        case 4: launch_fwd_sort<4>(ctx, f, blocks); break;
        case 8: launch_fwd_sort<8>(ctx, f, blocks); break;
        case 16: launch_fwd_sort<16>(ctx, f, blocks); break;
        case 32: launch_fwd_sort<32>(ctx, f, blocks); break;
        default: launch_fwd_sort<64>(ctx, f, blocks); break;
        }
        FAE_LAUNCH_CHECK(ctx);
    }
    ctx->presort.valid = true;
    ctx->presort.side = false;
    ctx->presort.ws = ws;
    ctx->presort.first_indices = hot_batch->h_indices[0];
    ctx->presort.n_samples = hot_batch->n_samples;
    ctx->presort.n_lookups = su.plan.N;
    ctx->presort.cur = 0;
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
    if (ctx->presort.valid && ctx->presort.side) {
        // whatever the side stream was asked to do must be finished before this workspace is used
        FAE_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->ev_join, 0));
    }
    if (ctx->presort.valid && ctx->presort.ws == ws && ctx->presort.first_indices == hot_batch->h_indices[0] &&
        ctx->presort.n_samples == hot_batch->n_samples && ctx->presort.n_lookups == plan.N) {
        cur = ctx->presort.cur;
    } else {
        rc = bwd_sort_stage(ctx, ctx->stream, hot_tables, hot_batch, su, &cur);
        if (rc != FAE_OK)
            return rc;
    }
    ctx->presort.valid = false;
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
        const bool scan_form = ctx->opt_reduce != 2 || a.mean || a.adagrad;
        a.fused_fixup = ctx->opt_fixup != 1 && scan_form && ncols <= lpr && spans <= a.n_flags;
#define CALL_REDUCE(V, L) launch_reduce<V, L>(ctx, a)
        if (vec) {
            BWD_LPR_SWITCH(float4, lpr, CALL_REDUCE)
        } else {
            BWD_LPR_SWITCH(float, lpr, CALL_REDUCE)
        }
#undef CALL_REDUCE
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
        hipLaunchKernelGGL(dbg_count_kernel, dim3((unsigned)plan.dbg_tiles), dim3(256), 0, ctx->stream, a);
        FAE_LAUNCH_CHECK(ctx);
        rc = fae_scan_i32(ctx, w.dbg_tile_sums, plan.dbg_tiles);
        if (rc != FAE_OK)
            return rc;
        hipLaunchKernelGGL(dbg_emit_kernel, dim3((unsigned)plan.dbg_tiles), dim3(256), 0, ctx->stream, a);
        FAE_LAUNCH_CHECK(ctx);
        int rl_blocks = (int)((plan.N + 255) / 256);
        if (rl_blocks > 4096)
            rl_blocks = 4096;
        hipLaunchKernelGGL(dbg_runlen_kernel, dim3(rl_blocks), dim3(256), 0, ctx->stream, a);
        FAE_LAUNCH_CHECK(ctx);
    }
    return FAE_OK;
}
