// Shared by the translation units of the backward (sort stage, reduce stage, entry points):
// geometry, kernel argument blocks, workspace layout, and the host functions that cross files.
#pragma once

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
    int32_t *ticket;   // [SWEEP_MAX_PASSES] next tile to hand out, per pass (use_ticket only)
    int32_t use_ticket; // chained passes: tiles are handed out by a counter instead of by workgroup number
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
    int32_t handoff;     // how border sums pass between workgroups: 0 device-scope accesses + wave-level ordering, 1 device-scope fences
    int32_t wg_waves;    // waves (spans) per workgroup of the reduce kernel: 1, 2 or 4
    int32_t form;        // reduce kernel: 0 scan across the lane groups, 1 a share of the span per lane group
    int32_t span;      // lookups per wave in the reduce kernel
    int32_t n_spans;   // total spans (blk_start then holds the span prefix per table)
    uint32_t *status;
    // debug outputs
    int32_t *dbg_uniq, *dbg_runlen, *dbg_table_start, *dbg_tile_sums, *dbg_rstart;
    int32_t dbg_tiles;
};

#define KEYS_PER_THREAD 4
#define KEYS_PER_BLOCK (256 * KEYS_PER_THREAD)
#define SWEEP_MAX_PASSES 4
#define SWEEP_AGGREGATE 1u // the tile's own digit count is published
#define SWEEP_PREFIX 2u    // the count of this and all earlier tiles of the table is published
#define SWEEP_SPIN_LIMIT (1 << 22)

static_assert(sizeof(BwdArgs) <= 4096, "kernel arguments are passed by value");

// in-LDS sort of small tables (also a role of the fused forward + sort kernel)
struct LsortArgs {
    const int32_t *slots[FAE_MAX_TABLES];
    const int32_t *offsets[FAE_MAX_TABLES];
    int32_t n_hot[FAE_MAX_TABLES];
    int32_t seg_start[FAE_MAX_TABLES + 1];
    int32_t blk_start[FAE_MAX_TABLES + 1]; // workgroups per table (0 for tables sorted elsewhere)
    int32_t part_shift[FAE_MAX_TABLES];    // part of a key = key >> part_shift
    int32_t n_tables;
    int32_t n_samples;
    int32_t unordered; // counting sort: the order inside a slot's run is left to the hardware
    int32_t *keys_out, *vals_out;
    uint32_t *status;
    int32_t *flags; // span flags of the reduce kernel, zeroed here
    int32_t n_flags, flag_slice;
};

#ifdef __HIPCC__
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
#endif

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------
struct BwdPlan {
    int64_t N;
    int64_t tiles;
    int64_t small_tiles; // tiles of SORT_TILE_SMALL keys
    int64_t max_spans; // with the smallest span
    int64_t dbg_tiles;
};

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

// Common set-up of the backward: validation, workspace carving, per-table descriptors.
struct BwdSetup {
    BwdPlan plan;
    BwdWs w;
    BwdArgs a;
    bool empty;
};

// fae_bwd.hip
BwdPlan bwd_plan(int nt, const int64_t *h_n_lookups);
int bwd_span(const BwdPlan &p, int n_cu);
BwdWs bwd_carve(void *ws, size_t bytes, const BwdPlan &p, int nt, int dim, int span);
int32_t bwd_setup(fae_ctx *ctx, const fae_tables *hot_tables, const fae_batch *hot_batch, void *ws, size_t ws_bytes,
                  const char *who, BwdSetup *out);
// fae_bwd_sort.hip: steps 1 + 2 on stream `st`; *cur_out names the ping-pong buffer with the result
int32_t bwd_sort_stage(fae_ctx *ctx, hipStream_t st, const fae_tables *hot_tables, const fae_batch *hot_batch,
                       BwdSetup &su, int *cur_out);
// fae_bwd_reduce.hip: steps 3 + 4 on the context's stream (vec: 16-byte column slices; lpr: lanes per row)
void bwd_launch_reduce(fae_ctx *ctx, const BwdArgs &a, bool vec, int lpr);
// fae_bwd_reduce.hip: distinct slots per table and their multiplicities (optional outputs of the backward)
int32_t bwd_launch_debug(fae_ctx *ctx, BwdArgs &a);
