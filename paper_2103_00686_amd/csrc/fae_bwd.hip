// Hot mini-batch backward + sparse SGD (Sec. 2.2 "optimizer on embeddings", Sec. 6.2:
// embedding update on the GPU for hot mini-batches).
//
//   1. keys      key = hot slot, value = sample id, per table segment
//   2. sort      stable LSD radix sort of (key, value), segmented by table; only the
//                bits a hot slot can occupy are sorted
//   3. reduce    a lane group walks a chunk of the sorted lookups, sums the upstream
//                gradient rows of each run of equal keys that STARTS in its chunk and
//                applies w -= lr * G once per distinct row (no float atomics: every
//                row has exactly one writer, sums follow sorted order)
//   4. long runs runs longer than BWD_LONG are cut into pieces, summed by one
//                workgroup per piece, then combined in piece order
// Bandwidth bound: per lookup one gradient row is read, per distinct row one weight
// row is read and written; the sort moves 16 B per lookup and pass.
#include "fae_internal.h"

// ---------------------------------------------------------------------------------
// sort geometry
// ---------------------------------------------------------------------------------
#define SORT_THREADS 256
#define SORT_ITEMS 16
#define SORT_WAVES (SORT_THREADS / FAE_WAVE)
#define SORT_TILE (SORT_THREADS * SORT_ITEMS)
#define RADIX_BITS 8
#define RADIX (1 << RADIX_BITS)

#define BWD_CHUNK 32    // sorted lookups per lane group in the reduce kernel
#define BWD_LONG 128    // a run with more elements than this is handled by the long-run kernels
#define BWD_PIECE 1024  // elements of a long run summed by one workgroup
#define DBG_TILE 2048

struct LongRun {
    int32_t z, key, start, end, piece_base, n_pieces;
};
struct Piece {
    int32_t run, beg, end;
};

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
    const float *gout;
    int64_t gout_stride;
    float lr;
    LongRun *longq;
    Piece *pieces;
    float *partial;
    int32_t *counters; // [0] long runs, [1] pieces
    int32_t long_cap, piece_cap;
    uint32_t *status;
    // debug outputs
    int32_t *dbg_uniq, *dbg_runlen, *dbg_table_start, *dbg_tile_sums, *dbg_rstart;
    int32_t dbg_tiles;
};

// ---------------------------------------------------------------------------------
// 1. keys
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bwd_keys_kernel(BwdArgs a)
{
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int j = (blockIdx.x - a.blk_start[z]) * 256 + threadIdx.x;
    const int n = a.seg_start[z + 1] - a.seg_start[z];
    if (j >= n)
        return;
    const int32_t *off = a.offsets[z];
    int s = off ? fae_sample_of(off, a.n_samples, j) : j;
    int k = a.slots[z][j];
    if ((unsigned)k >= (unsigned)a.n_hot[z]) {
        fae_flag(a.status, FAE_STATUS_ERANGE);
        k = a.n_hot[z]; // sorts behind every valid slot of the table; never dereferenced
    }
    if (off && (off[s] > j || off[s + 1] <= j))
        fae_flag(a.status, FAE_STATUS_ERANGE); // malformed CSR
    a.keys_in[a.seg_start[z] + j] = k;
    a.vals_in[a.seg_start[z] + j] = s;
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
#pragma unroll
    for (int i = 0; i < SORT_ITEMS; ++i) {
        int p = base + i * SORT_THREADS + threadIdx.x;
        if (p < seg1)
            atomicAdd(&cnt[(a.keys_in[p] >> a.shift) & a.mask], 1);
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

__global__ __launch_bounds__(SORT_THREADS) void sort_scatter_kernel(BwdArgs a)
{
    __shared__ int wcnt[SORT_WAVES][RADIX];
    __shared__ int digoff[SORT_WAVES][RADIX];
    __shared__ int scan_lds[SORT_THREADS / FAE_WAVE + 1];
    const int z = fae_find_table(a.tile_start, a.n_tables, blockIdx.x);
    const int tl = blockIdx.x - a.tile_start[z];
    const int tiles_z = a.tile_start[z + 1] - a.tile_start[z];
    const int seg1 = a.seg_start[z + 1];
    const int w = threadIdx.x / FAE_WAVE, lane = fae_lane();
    const int base = a.seg_start[z] + tl * SORT_TILE + w * (FAE_WAVE * SORT_ITEMS);
    volatile int *my_cnt = wcnt[w];
#pragma unroll
    for (int i = 0; i < RADIX / FAE_WAVE; ++i)
        my_cnt[i * FAE_WAVE + lane] = 0;
    __builtin_amdgcn_wave_barrier();

    int key[SORT_ITEMS], val[SORT_ITEMS], off[SORT_ITEMS];
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int i = 0; i < SORT_ITEMS; ++i) {
        const int p = base + i * FAE_WAVE + lane;
        const bool valid = p < seg1;
        key[i] = valid ? a.keys_in[p] : 0;
        val[i] = valid ? a.vals_in[p] : 0;
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
        // thread t owns digit t: offsets of the four waves inside this tile, plus the global base
        const int t = threadIdx.x;
        int c0 = wcnt[0][t], c1 = wcnt[1][t], c2 = wcnt[2][t];
        int total;
        int ex = fae_block_excl_scan<SORT_THREADS>(a.tot[z * RADIX + t], scan_lds, &total);
        int gb = a.seg_start[z] + ex + a.hist[RADIX * a.tile_start[z] + t * tiles_z + tl];
        digoff[0][t] = gb;
        digoff[1][t] = gb + c0;
        digoff[2][t] = gb + c0 + c1;
        digoff[3][t] = gb + c0 + c1 + c2;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < SORT_ITEMS; ++i) {
        const int p = base + i * FAE_WAVE + lane;
        if (p < seg1) {
            const int d = (key[i] >> a.shift) & a.mask;
            const int dst = digoff[w][d] + off[i];
            a.keys_out[dst] = key[i];
            a.vals_out[dst] = val[i];
        }
    }
}

// ---------------------------------------------------------------------------------
// 3. segment reduce + SGD for runs that start inside a chunk
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
};
template <> struct bwd_vec<float> {
    static __device__ __forceinline__ float zero() { return 0.f; }
    static __device__ __forceinline__ void add(float &a, const float &b) { a += b; }
    static __device__ __forceinline__ float sgd(const float &w, const float &g, float lr) { return w - lr * g; }
};

template <typename V, int LPR> __global__ __launch_bounds__(256) void bwd_reduce_kernel(BwdArgs a)
{
    constexpr int GPB = 256 / LPR;
    constexpr int VW = sizeof(V) / sizeof(float);
    const int z = fae_find_table(a.blk_start, a.n_tables, blockIdx.x);
    const int bl = blockIdx.x - a.blk_start[z];
    const int g = threadIdx.x / LPR, l = threadIdx.x % LPR;
    const int seg0 = a.seg_start[z], seg1 = a.seg_start[z + 1];
    const int64_t chunk = (int64_t)bl * GPB + g;
    const int64_t pos0_64 = seg0 + chunk * BWD_CHUNK;
    if (pos0_64 >= seg1)
        return;
    const int pos0 = (int)pos0_64;
    const int pos1 = pos0 + BWD_CHUNK < seg1 ? pos0 + BWD_CHUNK : seg1;
    const int ncols = a.dim / VW;
    const int n_hot = a.n_hot[z];
    const int32_t *keys = a.keys_in, *vals = a.vals_in;
    V *W = (V *)a.W[z];
    const float *gbase = a.gout + (int64_t)z * a.dim;
    for (int c0 = 0; c0 < ncols; c0 += LPR) {
        const int c = c0 + l;
        const bool active = c < ncols;
        int p = pos0;
        if (p > seg0) { // a run that began in an earlier chunk belongs to that chunk
            const int kprev = keys[p - 1];
            while (p < pos1 && keys[p] == kprev)
                ++p;
        }
        while (p < pos1) {
            const int k = keys[p];
            if (k >= n_hot) { // invalid slots (flagged when the keys were built) end the segment
                p = pos1;
                break;
            }
            if (p + BWD_LONG < seg1 && keys[p + BWD_LONG] == k) {
                if (l == 0 && c0 == 0) {
                    int q = atomicAdd(&a.counters[0], 1);
                    if (q < a.long_cap) {
                        LongRun r;
                        r.z = z;
                        r.key = k;
                        r.start = p;
                        r.end = 0;
                        r.piece_base = 0;
                        r.n_pieces = 0;
                        a.longq[q] = r;
                    }
                }
                ++p;
                while (p < pos1 && keys[p] == k)
                    ++p;
                continue;
            }
            V acc = bwd_vec<V>::zero();
            int q = p;
            do {
                const int s = vals[q];
                if (active)
                    bwd_vec<V>::add(acc, ((const V *)(gbase + (int64_t)s * a.gout_stride))[c]);
                ++q;
            } while (q < seg1 && keys[q] == k);
            if (active) {
                V *wp = W + (int64_t)k * ncols + c;
                *wp = bwd_vec<V>::sgd(*wp, acc, a.lr);
            }
            p = q;
        }
    }
}

// ---------------------------------------------------------------------------------
// 4. long runs
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bwd_long_prep_kernel(BwdArgs a)
{
    int n_long = a.counters[0];
    if (n_long > a.long_cap)
        n_long = a.long_cap;
    for (int q = blockIdx.x * 256 + threadIdx.x; q < n_long; q += gridDim.x * 256) {
        LongRun r = a.longq[q];
        const int seg1 = a.seg_start[r.z + 1];
        r.end = fae_upper_bound(a.keys_in, r.start, seg1, r.key);
        r.n_pieces = (r.end - r.start + BWD_PIECE - 1) / BWD_PIECE;
        r.piece_base = atomicAdd(&a.counters[1], r.n_pieces);
        for (int i = 0; i < r.n_pieces; ++i) {
            if (r.piece_base + i < a.piece_cap) {
                Piece pc;
                pc.run = q;
                pc.beg = r.start + i * BWD_PIECE;
                pc.end = pc.beg + BWD_PIECE < r.end ? pc.beg + BWD_PIECE : r.end;
                a.pieces[r.piece_base + i] = pc;
            }
        }
        a.longq[q] = r;
    }
}

// one workgroup per piece: lane groups take alternate rows, then are summed in group order
template <typename V, int LPR> __global__ __launch_bounds__(256) void bwd_long_piece_kernel(BwdArgs a)
{
    constexpr int G = 256 / LPR;
    constexpr int VW = sizeof(V) / sizeof(float);
    __shared__ V red[256];
    int n_pieces = a.counters[1];
    if (n_pieces > a.piece_cap)
        n_pieces = a.piece_cap;
    const int g = threadIdx.x / LPR, l = threadIdx.x % LPR;
    const int ncols = a.dim / VW;
    for (int pi = blockIdx.x; pi < n_pieces; pi += gridDim.x) {
        const Piece pc = a.pieces[pi];
        const int z = a.longq[pc.run].z;
        const float *gbase = a.gout + (int64_t)z * a.dim;
        for (int c0 = 0; c0 < ncols; c0 += LPR) {
            const int c = c0 + l;
            V acc = bwd_vec<V>::zero();
            if (c < ncols) {
                int q = pc.beg + g;
                for (; q + 3 * G < pc.end; q += 4 * G) {
                    const int s0 = a.vals_in[q], s1 = a.vals_in[q + G], s2 = a.vals_in[q + 2 * G], s3 = a.vals_in[q + 3 * G];
                    const V v0 = ((const V *)(gbase + (int64_t)s0 * a.gout_stride))[c];
                    const V v1 = ((const V *)(gbase + (int64_t)s1 * a.gout_stride))[c];
                    const V v2 = ((const V *)(gbase + (int64_t)s2 * a.gout_stride))[c];
                    const V v3 = ((const V *)(gbase + (int64_t)s3 * a.gout_stride))[c];
                    bwd_vec<V>::add(acc, v0);
                    bwd_vec<V>::add(acc, v1);
                    bwd_vec<V>::add(acc, v2);
                    bwd_vec<V>::add(acc, v3);
                }
                for (; q < pc.end; q += G)
                    bwd_vec<V>::add(acc, ((const V *)(gbase + (int64_t)a.vals_in[q] * a.gout_stride))[c]);
            }
            __syncthreads(); // red may still be read from the previous column block / piece
            red[threadIdx.x] = acc;
            __syncthreads();
            if (g == 0 && c < ncols) {
                V sum = red[l];
                for (int gg = 1; gg < G; ++gg)
                    bwd_vec<V>::add(sum, red[gg * LPR + l]);
                ((V *)(a.partial + (int64_t)pi * a.dim))[c] = sum;
            }
        }
    }
}

// one lane group per long run: pieces are combined in order, then one SGD update
template <typename V, int LPR> __global__ __launch_bounds__(256) void bwd_long_final_kernel(BwdArgs a)
{
    constexpr int GPB = 256 / LPR;
    constexpr int VW = sizeof(V) / sizeof(float);
    int n_long = a.counters[0];
    if (n_long > a.long_cap)
        n_long = a.long_cap;
    const int g = threadIdx.x / LPR, l = threadIdx.x % LPR;
    const int ncols = a.dim / VW;
    for (int q = blockIdx.x * GPB + g; q < n_long; q += gridDim.x * GPB) {
        const LongRun r = a.longq[q];
        if (r.piece_base + r.n_pieces > a.piece_cap)
            continue; // cannot happen with the documented workspace size
        for (int c = l; c < ncols; c += LPR) {
            V acc = bwd_vec<V>::zero();
            for (int i = 0; i < r.n_pieces; ++i)
                bwd_vec<V>::add(acc, ((const V *)(a.partial + (int64_t)(r.piece_base + i) * a.dim))[c]);
            V *wp = (V *)a.W[r.z] + (int64_t)r.key * ncols + c;
            *wp = bwd_vec<V>::sgd(*wp, acc, a.lr);
        }
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
    int64_t long_cap, piece_cap;
    int64_t dbg_tiles;
};

BwdPlan bwd_plan(int nt, const int64_t *h_n_lookups)
{
    BwdPlan p;
    p.N = 0;
    p.tiles = 0;
    for (int z = 0; z < nt; ++z) {
        p.N += h_n_lookups[z];
        p.tiles += (h_n_lookups[z] + SORT_TILE - 1) / SORT_TILE;
    }
    p.long_cap = p.N / (BWD_LONG + 1) + 1;
    p.piece_cap = p.N / BWD_PIECE + p.long_cap + 1;
    p.dbg_tiles = (p.N + DBG_TILE - 1) / DBG_TILE;
    return p;
}

struct BwdWs {
    int32_t *keys[2], *vals[2];
    int32_t *hist, *tot, *counters;
    LongRun *longq;
    Piece *pieces;
    float *partial;
    int32_t *dbg_tile_sums, *dbg_rstart;
    bool ok;
    size_t used;
};

BwdWs bwd_carve(void *ws, size_t bytes, const BwdPlan &p, int nt, int dim)
{
    fae_carver cv(ws, bytes);
    BwdWs w;
    for (int i = 0; i < 2; ++i) {
        w.keys[i] = cv.take<int32_t>((size_t)p.N + 1);
        w.vals[i] = cv.take<int32_t>((size_t)p.N + 1);
    }
    w.hist = cv.take<int32_t>((size_t)RADIX * p.tiles + 1);
    w.tot = cv.take<int32_t>((size_t)nt * RADIX);
    w.counters = cv.take<int32_t>(64);
    w.longq = cv.take<LongRun>((size_t)p.long_cap);
    w.pieces = cv.take<Piece>((size_t)p.piece_cap);
    w.partial = cv.take<float>((size_t)p.piece_cap * dim);
    w.dbg_tile_sums = cv.take<int32_t>((size_t)p.dbg_tiles + 2);
    w.dbg_rstart = cv.take<int32_t>((size_t)p.N + 2);
    w.ok = cv.ok;
    w.used = cv.used;
    return w;
}

template <typename V, int LPR> void launch_reduce(fae_ctx *ctx, const BwdArgs &a, int blocks)
{
    hipLaunchKernelGGL((bwd_reduce_kernel<V, LPR>), dim3(blocks), dim3(256), 0, ctx->stream, a);
}
template <typename V, int LPR> void launch_long(fae_ctx *ctx, const BwdArgs &a, int piece_blocks, int final_blocks)
{
    {
        fae_ktimer kt(ctx, FAE_K_LONG_PIECE);
        hipLaunchKernelGGL((bwd_long_piece_kernel<V, LPR>), dim3(piece_blocks), dim3(256), 0, ctx->stream, a);
    }
    fae_ktimer kt(ctx, FAE_K_LONG_FINAL);
    hipLaunchKernelGGL((bwd_long_final_kernel<V, LPR>), dim3(final_blocks), dim3(256), 0, ctx->stream, a);
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
    BwdWs w = bwd_carve((void *)256, (size_t)-1, p, hot_tables->n_tables, hot_tables->dim);
    return w.used + 256;
}

extern "C" int32_t fae_embbag_bwd_sgd(fae_ctx *ctx, const fae_tables *hot_tables, float *const *h_hotW,
                                      const fae_batch *hot_batch, const float *gout, int64_t gout_row_stride,
                                      float lr, const fae_bwd_debug *dbg, void *ws, size_t ws_bytes)
{
    int32_t rc = fae_check_tables(ctx, hot_tables, "fae_embbag_bwd_sgd");
    if (rc != FAE_OK)
        return rc;
    rc = fae_check_batch(ctx, hot_tables, hot_batch, "fae_embbag_bwd_sgd");
    if (rc != FAE_OK)
        return rc;
    const int nt = hot_tables->n_tables, dim = hot_tables->dim;
    if (dbg && !dbg->table_start)
        return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_sgd: incomplete debug outputs");
    const int64_t S = hot_batch->n_samples;
    const BwdPlan plan = bwd_plan(nt, hot_batch->h_n_lookups);
    if (plan.N >= 2147483647LL - SORT_TILE)
        return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_sgd: more than 2^31 lookups in one call");
    FAE_HIP(ctx, hipSetDevice(ctx->device));
    if (plan.N == 0 || S == 0) { // nothing to update
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
    if (!ws)
        return fae_fail(ctx, FAE_ENOSPC, "fae_embbag_bwd_sgd: null workspace");
    BwdWs w = bwd_carve(ws, ws_bytes, plan, nt, dim);
    if (!w.ok)
        return fae_fail(ctx, FAE_ENOSPC, "fae_embbag_bwd_sgd: workspace too small (%zu needed)", w.used);

    BwdArgs a;
    memset(&a, 0, sizeof(a));
    bool vec = (dim % 4 == 0) && (gout_row_stride % 4 == 0) && (((uintptr_t)gout) % 16 == 0);
    int64_t max_hot = 0;
    int64_t lookups = 0, tiles = 0;
    for (int z = 0; z < nt; ++z) {
        if (!h_hotW[z] && hot_tables->h_rows[z] > 0)
            return fae_fail(ctx, FAE_EINVAL, "fae_embbag_bwd_sgd: null weights for table %d", z);
        a.W[z] = h_hotW[z];
        a.slots[z] = hot_batch->h_indices[z];
        a.offsets[z] = hot_batch->h_offsets ? hot_batch->h_offsets[z] : nullptr;
        a.n_hot[z] = (int32_t)hot_tables->h_rows[z];
        if (((uintptr_t)h_hotW[z]) % 16 != 0)
            vec = false;
        if (hot_tables->h_rows[z] > max_hot)
            max_hot = hot_tables->h_rows[z];
        a.seg_start[z] = (int32_t)lookups;
        a.tile_start[z] = (int32_t)tiles;
        lookups += hot_batch->h_n_lookups[z];
        tiles += (hot_batch->h_n_lookups[z] + SORT_TILE - 1) / SORT_TILE;
    }
    a.seg_start[nt] = (int32_t)lookups;
    a.tile_start[nt] = (int32_t)tiles;
    a.n_tables = nt;
    a.dim = dim;
    a.n_samples = (int32_t)S;
    a.hist = w.hist;
    a.tot = w.tot;
    a.gout = gout;
    a.gout_stride = gout_row_stride;
    a.lr = lr;
    a.longq = w.longq;
    a.pieces = w.pieces;
    a.partial = w.partial;
    a.counters = w.counters;
    a.long_cap = (int32_t)plan.long_cap;
    a.piece_cap = (int32_t)plan.piece_cap;
    a.status = ctx->d_block;

    // 1. keys (also clears the long-run counters for this call)
    rc = fae_fill_u32(ctx, w.counters, 64, 0u);
    if (rc != FAE_OK)
        return rc;
    {
        int64_t blocks = 0;
        for (int z = 0; z < nt; ++z) {
            a.blk_start[z] = (int32_t)blocks;
            blocks += (hot_batch->h_n_lookups[z] + 255) / 256;
        }
        a.blk_start[nt] = (int32_t)blocks;
        a.keys_in = w.keys[0];
        a.vals_in = w.vals[0];
        fae_ktimer kt(ctx, FAE_K_BWD_KEYS);
        hipLaunchKernelGGL(bwd_keys_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, a);
        FAE_LAUNCH_CHECK(ctx);
    }
    // 2. sort: only the bits a slot (or the invalid marker n_hot) can occupy
    int bits = 1;
    while ((max_hot >> bits) != 0)
        ++bits;
    const int passes = (bits + RADIX_BITS - 1) / RADIX_BITS;
    const int digit_bits = (bits + passes - 1) / passes;
    int cur = 0;
    for (int pass = 0; pass < passes; ++pass) {
        a.shift = pass * digit_bits;
        a.mask = (1 << digit_bits) - 1;
        a.keys_in = w.keys[cur];
        a.vals_in = w.vals[cur];
        a.keys_out = w.keys[cur ^ 1];
        a.vals_out = w.vals[cur ^ 1];
        {
            fae_ktimer kt(ctx, FAE_K_SORT_HIST);
            hipLaunchKernelGGL(sort_hist_kernel, dim3((unsigned)tiles), dim3(SORT_THREADS), 0, ctx->stream, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        {
            fae_ktimer kt(ctx, FAE_K_SORT_COLSCAN);
            hipLaunchKernelGGL(sort_colscan_kernel, dim3((unsigned)((nt * RADIX + 3) / 4)), dim3(256), 0, ctx->stream, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        {
            fae_ktimer kt(ctx, FAE_K_SORT_SCATTER);
            hipLaunchKernelGGL(sort_scatter_kernel, dim3((unsigned)tiles), dim3(SORT_THREADS), 0, ctx->stream, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        cur ^= 1;
    }
    a.keys_in = w.keys[cur];
    a.vals_in = w.vals[cur];
    a.keys_out = nullptr;
    a.vals_out = nullptr;

    // 3. reduce + SGD
    const int ncols = vec ? dim / 4 : dim;
    int lpr = 1;
    while (lpr < ncols && lpr < 64)
        lpr <<= 1;
    {
        const int gpb = 256 / lpr;
        int64_t blocks = 0;
        for (int z = 0; z < nt; ++z) {
            a.blk_start[z] = (int32_t)blocks;
            int64_t chunks = (hot_batch->h_n_lookups[z] + BWD_CHUNK - 1) / BWD_CHUNK;
            blocks += (chunks + gpb - 1) / gpb;
        }
        a.blk_start[nt] = (int32_t)blocks;
        const int nb = (int)blocks;
        fae_ktimer kt(ctx, FAE_K_BWD_REDUCE);
#define CALL_REDUCE(V, L) launch_reduce<V, L>(ctx, a, nb)
        if (vec) {
            BWD_LPR_SWITCH(float4, lpr, CALL_REDUCE)
        } else {
            BWD_LPR_SWITCH(float, lpr, CALL_REDUCE)
        }
#undef CALL_REDUCE
        FAE_LAUNCH_CHECK(ctx);
    }
    // 4. long runs
    {
        int prep_blocks = (int)((plan.long_cap + 255) / 256);
        if (prep_blocks > 256)
            prep_blocks = 256;
        {
            fae_ktimer kt(ctx, FAE_K_LONG_PREP);
            hipLaunchKernelGGL(bwd_long_prep_kernel, dim3(prep_blocks), dim3(256), 0, ctx->stream, a);
            FAE_LAUNCH_CHECK(ctx);
        }
        int piece_blocks = (int)(plan.piece_cap < 4 * ctx->n_cu ? plan.piece_cap : 4 * ctx->n_cu);
        int final_blocks = (int)((plan.long_cap + (256 / lpr) - 1) / (256 / lpr));
        if (final_blocks > 2 * ctx->n_cu)
            final_blocks = 2 * ctx->n_cu;
#define CALL_LONG(V, L) launch_long<V, L>(ctx, a, piece_blocks, final_blocks)
        if (vec) {
            BWD_LPR_SWITCH(float4, lpr, CALL_LONG)
        } else {
            BWD_LPR_SWITCH(float, lpr, CALL_LONG)
        }
#undef CALL_LONG
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
