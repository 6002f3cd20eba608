// Backward, steps 1 + 2: (hot slot, sample) pairs of a hot mini-batch sorted by slot, per table
// (Sec. 2.2, Sec. 6.2: the embedding update of hot mini-batches runs on the GPU).
//   keys     key = hot slot, value = sample id, per table segment
//   sort     inside LDS for tables of up to 16 K lookups (split over workgroups by key range),
//            else stable LSD radix passes over only the bits a hot slot can occupy: one chained
//            kernel per pass for short lists, histogram / column scan / scatter for long ones
// Also here: the sort started ahead of the backward (side stream), and the launch that carries
// the forward's row copies and the LDS sort together.
#include "fae_bwd.h"

// ---------------------------------------------------------------------------------
// 1. keys
// ---------------------------------------------------------------------------------

// Four consecutive lookups of one thread: (slot, sample) pairs, 16-byte loads and stores when
// aligned, plus the digit counts of every radix pass into the workgroup's LDS histograms.
// vs: the samples of the four lookups (tables with offsets; else a lookup is its own sample).
__device__ __forceinline__ void bwd_keys_thread(const BwdArgs &a, int z, int j0, int n, const int32_t *off, const int *vs,
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
#pragma unroll
    for (int q = 0; q < KEYS_PER_THREAD; ++q) {
        const int j = j0 + q;
        v[q] = j;
        if (j >= n)
            continue;
        if ((unsigned)k[q] >= (unsigned)a.n_hot[z]) {
            bad = true;
            k[q] = a.n_hot[z]; // sorts behind every valid slot of the table; never dereferenced
        }
        if (off) {
            v[q] = vs[q]; // inside [0, n_samples) whatever the offsets hold
            if (off[v[q]] > j || off[v[q] + 1] <= j)
                bad = true; // malformed CSR
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

// how many of the workgroup's threads hold `flag` (every thread calls it; red: 256 / 64 + 1 ints)
__device__ __forceinline__ int keys_block_count(bool flag, int *red)
{
    const int c = __popcll(__ballot(flag));
    __syncthreads(); // red may still be read from a previous call
    if (fae_lane() == 0)
        red[threadIdx.x / FAE_WAVE] = c;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// Each thread handles four consecutive lookups (16-byte loads and stores when aligned).
// Tables with offsets: which sample a lookup belongs to is found by the workgroup together.
//   1. the sample of the workgroup's first lookup: an upper-bound search over the offsets in
//      which every round probes 256 evenly spaced entries at once (three dependent loads for
//      65 536 samples, where a search by one thread makes seventeen);
//   2. every later bag that starts among the workgroup's 1024 lookups marks its first lookup
//      with its sample number (the largest one wins where empty bags share a start);
//   3. a running maximum over the marks gives every lookup its sample.
__global__ __launch_bounds__(256) void bwd_keys_kernel(BwdArgs a)
{
    static_assert(KEYS_PER_BLOCK == 256 * KEYS_PER_THREAD, "one workgroup of 256 threads per block of lookups");
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int jb = (blockIdx.x - a.blk_start[z]) * KEYS_PER_BLOCK; // the workgroup's first lookup (inside the table)
    const int j0 = jb + threadIdx.x * KEYS_PER_THREAD;
    const int n = a.seg_start[z + 1] - a.seg_start[z];
    const int32_t *off = a.offsets[z];
    __shared__ int s_hist[SWEEP_MAX_PASSES][RADIX];
    __shared__ int s_mark[KEYS_PER_BLOCK];
    __shared__ int s_red[256 / FAE_WAVE + 1];
    for (int p = 0; p < a.n_passes; ++p)
        s_hist[p][threadIdx.x] = 0;
    int vs[KEYS_PER_THREAD] = {0, 0, 0, 0};
    if (off) {
        const int jend = jb + KEYS_PER_BLOCK < n ? jb + KEYS_PER_BLOCK : n;
#pragma unroll
        for (int q = 0; q < KEYS_PER_THREAD; ++q)
            s_mark[threadIdx.x * KEYS_PER_THREAD + q] = -1;
        // 1. entries of offsets[0 .. n_samples] that are <= jb: all before lo are, none from hi on is
        int lo = 0, hi = a.n_samples + 1;
        while (hi - lo > 256) {
            const int step = (hi - lo + 255) / 256;
            const int64_t idx = (int64_t)lo + (int64_t)(threadIdx.x + 1) * step - 1; // last entry of piece threadIdx.x
            const bool le = idx < hi && off[idx] <= jb;
            const int c = keys_block_count(le, s_red); // pieces that lie wholly at or below jb
            lo += c * step;
            hi = lo + step < hi ? lo + step : hi;
        }
        const bool le = lo + (int)threadIdx.x < hi && off[lo + threadIdx.x] <= jb;
        int s_first = lo + keys_block_count(le, s_red) - 1;
        s_first = s_first < 0 ? 0 : (s_first >= a.n_samples ? a.n_samples - 1 : s_first);
        // 2. (also orders the clearing of s_mark above before the marks: keys_block_count has barriers)
        for (int64_t s = (int64_t)s_first + 1 + threadIdx.x; s < a.n_samples; s += 256) {
            const int o = off[s];
            if (o >= jend)
                break;
            if (o >= jb)
                atomicMax(&s_mark[o - jb], (int)s);
        }
        __syncthreads();
        // 3. inclusive running maximum, four positions per thread
        int m[KEYS_PER_THREAD];
        int own = -1;
#pragma unroll
        for (int q = 0; q < KEYS_PER_THREAD; ++q) {
            m[q] = s_mark[threadIdx.x * KEYS_PER_THREAD + q];
            own = own > m[q] ? own : m[q];
        }
        int run = own; // maximum over this and the earlier threads of the wave
#pragma unroll
        for (int d = 1; d < FAE_WAVE; d <<= 1) {
            const int o = __shfl_up(run, d, FAE_WAVE);
            if (fae_lane() >= d)
                run = run > o ? run : o;
        }
        __syncthreads(); // s_red was read by keys_block_count
        if (fae_lane() == FAE_WAVE - 1)
            s_red[threadIdx.x / FAE_WAVE] = run;
        __syncthreads();
        int before = s_first; // everything in front of this thread's positions
        for (int w = 0; w < (int)(threadIdx.x / FAE_WAVE); ++w)
            before = before > s_red[w] ? before : s_red[w];
        const int prev = __shfl_up(run, 1, FAE_WAVE);
        if (fae_lane() > 0)
            before = before > prev ? before : prev;
#pragma unroll
        for (int q = 0; q < KEYS_PER_THREAD; ++q) {
            before = before > m[q] ? before : m[q];
            vs[q] = before;
        }
    }
    __syncthreads();
    if (j0 < n)
        bwd_keys_thread(a, z, j0, n, off, vs, s_hist);
    if (a.n_passes > 0) {
        __syncthreads();
        for (int p = 0; p < a.n_passes; ++p) {
            const int c = s_hist[p][threadIdx.x];
            if (c)
                atomicAdd(&a.ghist[(z * SWEEP_MAX_PASSES + p) * RADIX + threadIdx.x], c);
        }
    }
}


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
// CHAINED = true : the whole pass is this one kernel.  A tile publishes its digit counts,
// then adds up the published counts of the tiles before it (walking back until it meets a
// tile that already published its running total) and publishes its own running total.  A
// tile only ever waits for tiles with smaller workgroup numbers, which the hardware starts
// first; the wait is bounded all the same and reports an internal error instead of spinning
// forever.  (Handing tiles out through a counter instead makes the order certain but costs
// ~35 ns per workgroup, one device-wide atomic after the other: half the time of a pass over
// a short list.  sort_variant 4 does it that way.)
template <bool CHAINED, int ITEMS> __global__ __launch_bounds__(SORT_THREADS) void sort_scatter_kernel(BwdArgs a)
{
    constexpr int TILE = SORT_THREADS * ITEMS;
    __shared__ int wcnt[SORT_WAVES][RADIX];  // per wave: running count, then start inside the tile
    __shared__ int gbase[RADIX];             // global position of the tile's first element of a digit
    __shared__ int tbase[RADIX];             // position inside the tile of the first element of a digit
    __shared__ int skey[TILE], sval[TILE];
    __shared__ int scan_lds[SORT_THREADS / FAE_WAVE + 1];
    __shared__ int s_tile;
    __shared__ int s_gave_up; // a chained wait of this tile gave up: nothing of the tile is written
    if (CHAINED && threadIdx.x == 0)
        s_gave_up = 0;
    int tile = blockIdx.x;
    if (CHAINED && a.use_ticket) {
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
                                s_gave_up = 1;
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
    // The running total of a tile whose wait gave up is wrong (it was published all the same, so
    // that later tiles do not wait in turn): its pairs are not written.  The status word is set;
    // the reduce kernel looks at it before it reads any pair and leaves the tables alone.
    if (CHAINED && s_gave_up)
        return;
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

__global__ __launch_bounds__(LSORT_THREADS) void lds_sort_kernel(LsortArgs a)
{
    bwd_clear_flags(a.flags, a.n_flags, a.flag_slice, LSORT_THREADS);
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    lds_sort_block(a.slots[z], a.offsets[z], a.seg_start[z + 1] - a.seg_start[z], a.n_hot[z],
                   blockIdx.x - a.blk_start[z], a.part_shift[z], a.n_samples, a.keys_out + a.seg_start[z],
                   a.vals_out + a.seg_start[z], a.status, a.unordered != 0);
}

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------
// Workgroups per small table for the LDS sort: enough parts to occupy the chip, never lists
// below ~512 lookups.  part_shift[z]: part of a key = key >> shift; blk_start: prefix of
// workgroups per table (tables not sorted in LDS get none).  Returns the number of workgroups.
static int lsort_plan(const fae_ctx *ctx, const fae_tables *hot_tables, const fae_batch *hot_batch, const bool *in_lds,
               int n_lds, int32_t *blk_start, int32_t *part_shift, int64_t other_blocks)
{
    const int nt = hot_tables->n_tables;
    int want = 1;
    while (want < 16 && n_lds * want * 2 <= ctx->n_cu)
        want <<= 1;
    // In the launch that also copies rows (other_blocks workgroups of them, one workgroup per
    // compute unit), every sorting workgroup keeps a unit from copying: when the copies alone are
    // more than the chip holds at once, fewer and larger parts win although the largest part ends
    // later (workload 3: 35.5 us with 4 parts per table, 38.9 us with 8, 43.5 us with 2).
    while (want > 4 && (int64_t)n_lds * want + other_blocks > (int64_t)ctx->n_cu * 3 / 2)
        want >>= 1;
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
        if (!in_lds[z] && nl > 0 && hot_tables->h_rows[z] > max_hot_global)
            max_hot_global = hot_tables->h_rows[z];
    }
    // When some table needs the global passes anyway, a small table whose slots need no more
    // passes than those rides along: its few tiles cost nothing there, and if no small table is
    // left the LDS sort (a launch of its own, ~10 us however small the table) is not needed.
    if (max_hot_global > 0 && ctx->opt_sort != 2) {
        int gbits = 1;
        while ((max_hot_global >> gbits) != 0)
            ++gbits;
        const int gpasses = (gbits + RADIX_BITS - 1) / RADIX_BITS;
        for (int z = 0; z < nt; ++z)
            if (in_lds[z] && hot_tables->h_rows[z] < (1LL << (gpasses * RADIX_BITS)))
                in_lds[z] = false;
    }
    for (int z = 0; z < nt; ++z) {
        const int64_t nl = hot_batch->h_n_lookups[z];
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
    const bool chained =
        passes > 0 && ctx->opt_sort != 1 && (ctx->opt_sort == 3 || ctx->opt_sort == 4 || tiles <= 4LL * ctx->n_cu);
    a.use_ticket = ctx->opt_sort == 4;
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
            FAE_LAUNCH(ctx, bwd_keys_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a);
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
                FAE_LAUNCH(ctx, (sort_scatter_kernel<true, SORT_ITEMS_SMALL>), dim3((unsigned)tiles), dim3(SORT_THREADS), 0, st, a);
            else
                FAE_LAUNCH(ctx, (sort_scatter_kernel<true, SORT_ITEMS>), dim3((unsigned)tiles), dim3(SORT_THREADS), 0, st, a);
            FAE_LAUNCH_CHECK(ctx);
            cur ^= 1;
            continue;
        }
        {
            fae_ktimer kt(ctx, FAE_K_SORT_HIST, st);
            FAE_LAUNCH(ctx, sort_hist_kernel, dim3((unsigned)tiles), dim3(SORT_THREADS), 0, st, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        {
            fae_ktimer kt(ctx, FAE_K_SORT_COLSCAN, st);
            FAE_LAUNCH(ctx, sort_colscan_kernel, dim3((unsigned)((nt * RADIX + 3) / 4)), dim3(256), 0, st, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        {
            fae_ktimer kt(ctx, FAE_K_SORT_SCATTER, st);
            FAE_LAUNCH(ctx, (sort_scatter_kernel<false, SORT_ITEMS>), dim3((unsigned)tiles), dim3(SORT_THREADS), 0, st, a);
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
        const int nb = lsort_plan(ctx, hot_tables, hot_batch, in_lds, n_lds, la.blk_start, la.part_shift, 0);
        la.seg_start[nt] = a.seg_start[nt];
        la.n_tables = nt;
        la.n_samples = a.n_samples;
        la.keys_out = w.keys[cur];
        la.vals_out = w.vals[cur];
        la.status = ctx->d_block;
        la.unordered = ctx->opt_sort_order == 1;
        la.flags = a.flags;
        la.n_flags = a.n_flags;
        la.flag_slice = bwd_flag_slice(a.n_flags, nb);
        fae_ktimer kt(ctx, FAE_K_LDS_SORT, st);
        FAE_LAUNCH(ctx, lds_sort_kernel, dim3(nb), dim3(LSORT_THREADS), 0, st, la);
        FAE_LAUNCH_CHECK(ctx);
    }
    *cur_out = cur;
    return FAE_OK;
}

extern "C" int32_t fae_embbag_bwd_presort(fae_ctx *ctx, const fae_tables *hot_tables, const fae_batch *hot_batch,
                                          void *ws, size_t ws_bytes)
{
    BwdSetup su;
    int32_t rc = bwd_setup(ctx, hot_tables, hot_batch, ws, ws_bytes, "fae_embbag_bwd_presort", &su);
    if (rc != FAE_OK)
        return rc;
    FAE_HIP(ctx, hipSetDevice(ctx->device));
    fae_ctx::Presort *ps = ctx->presort_slot(ws);
    if (ps->valid && ps->side) // an unused sort (of this workspace, or the oldest one): nothing else would wait for it
        FAE_HIP(ctx, hipStreamWaitEvent(ctx->stream, ps->ev_join, 0));
    ps->valid = false;
    if (su.empty)
        return FAE_OK;
    // fork: the side stream starts after everything already queued on the main stream
    // (earlier users of this workspace, producers of the slots)
    const int side = ctx->aux_next;
    ctx->aux_next = (side + 1) % fae_ctx::N_AUX;
    FAE_HIP(ctx, hipEventRecord(ctx->ev_fork[side], ctx->stream));
    FAE_HIP(ctx, hipStreamWaitEvent(ctx->aux_stream[side], ctx->ev_fork[side], 0));
    int cur = 0;
    rc = bwd_sort_stage(ctx, ctx->aux_stream[side], hot_tables, hot_batch, su, &cur);
    if (rc != FAE_OK)
        return rc;
    FAE_HIP(ctx, hipEventRecord(ps->ev_join, ctx->aux_stream[side]));
    ps->valid = true;
    ps->side = true;
    ps->ws = ws;
    fae_ctx::presort_bind(ps, hot_tables->n_tables, hot_batch);
    ps->cur = cur;
    ps->age = ++ctx->presort_clock;
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
    int32_t unordered;
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
                       a.vals_out + a.seg_start[z], a.status, a.unordered != 0);
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
    FAE_LAUNCH(ctx, (fwd_sort_kernel<float4, LPR>), dim3(blocks), dim3(LSORT_THREADS), 0, ctx->stream, a);
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
    fae_ctx::Presort *ps = ctx->presort_slot(ws);
    if (ps->valid && ps->side) // an unused sort (of this workspace, or the oldest one): nothing else would wait for it
        FAE_HIP(ctx, hipStreamWaitEvent(ctx->stream, ps->ev_join, 0));
    ps->valid = false;
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
    f.n_sort_blocks = lsort_plan(ctx, hot_tables, hot_batch, in_lds, nt, f.sort_blk_start, f.part_shift,
                                (int64_t)nt * ((S + LSORT_THREADS - 1) / LSORT_THREADS));
    f.n_tables = nt;
    f.dim = dim;
    f.n_samples = (int32_t)S;
    f.fwd_blocks_per_table = (int32_t)((S + LSORT_THREADS - 1) / LSORT_THREADS);
    f.out_stride = out_row_stride;
    f.out = out;
    f.keys_out = su.w.keys[0];
    f.vals_out = su.w.vals[0];
    f.status = ctx->d_block;
    f.unordered = ctx->opt_sort_order == 1;
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
    ps->valid = true;
    ps->side = false;
    ps->ws = ws;
    fae_ctx::presort_bind(ps, nt, hot_batch);
    ps->cur = 0;
    ps->age = ++ctx->presort_clock;
    return FAE_OK;
}
