/*
 * libfae -- the GPU-resident hot path of the FAE (Frequently Accessed Embeddings)
 * training method, arxiv 2103.00686, for AMD MI355X (gfx950).
 *
 * The path, in the paper's order (Sec. 4, Fig. 4 and Fig. 6):
 *   profile (Embedding Logger)  ->  cutoff (Eq. 1 / budget L)  ->  classify + remap +
 *   hot tables (Embedding Classifier, Embedding Replicator)  ->  partition (Input
 *   Classifier)  ->  hot mini-batch forward (sum-pooled embedding bags)  ->  backward
 *   (sort by row, sum duplicates)  ->  sparse SGD on the hot tables.
 *
 * Conventions
 *   - C ABI, no exceptions, no global state.  Every call returns FAE_OK (0) or a
 *     negative error code; fae_last_error() gives text for the last failure.
 *   - Pointers named h_* are HOST pointers (small arrays of per-table values or of
 *     per-table device pointers).  Every other pointer is a DEVICE pointer owned
 *     by the caller.  The library allocates no user-visible device memory: bulk
 *     scratch comes in through (ws, ws_bytes), sized by the *_workspace_bytes()
 *     queries.  A context owns only one 4 KiB device block and one 4 KiB pinned
 *     host block for status words and scalar read-backs.
 *   - All kernels are enqueued on the stream given to fae_create().  Calls are
 *     asynchronous unless documented as synchronising.
 *   - Index validation happens on the device: an index outside [0, rows), a slot
 *     outside [0, n_hot) or a malformed CSR is never dereferenced; it is skipped
 *     and a sticky status bit is set, which the next synchronising call (or
 *     fae_sync) returns as FAE_ERANGE / FAE_ENOSPC and then clears.
 *   - Types: row ids, hot slots, sample ids and CSR offsets are int32; access
 *     counts are uint32 (precondition: fewer than 2^32 accesses per row);
 *     weights, pooled outputs and gradients are fp32, row-major.
 *   - Limits: n_tables <= FAE_MAX_TABLES; dim >= 1 (dim % 4 == 0 takes the
 *     16-byte vector path); lookups per table per call < 2^31; rows per table < 2^31.
 */
#ifndef FAE_H
#define FAE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FAE_MAX_TABLES 64

#define FAE_OK 0
#define FAE_EINVAL (-1) /* bad argument (null pointer, size, limit)                 */
#define FAE_ERANGE (-2) /* index/slot out of range or malformed CSR (device-detected) */
#define FAE_ENOSPC (-3) /* workspace or output capacity too small                   */
#define FAE_EHIP   (-4) /* HIP runtime error; see fae_last_error()                  */

typedef struct fae_ctx fae_ctx;

/* Shape of a set of embedding tables: n_tables tables of h_rows[z] rows, all of
 * row dimension dim.  For hot tables, h_rows[z] is n_hot_z. */
typedef struct {
    int32_t n_tables;
    int32_t dim;
    const int64_t *h_rows; /* host, [n_tables] */
} fae_tables;

/* A chunk of sparse inputs: per table a CSR over samples, table-major.
 * h_offsets == NULL, or h_offsets[z] == NULL, means one lookup per sample in
 * table z (then h_n_lookups[z] must equal n_samples). */
typedef struct {
    int64_t n_samples;
    const int32_t *const *h_indices; /* host [n_tables] -> device int32[n_lookups_z]  */
    const int32_t *const *h_offsets; /* host [n_tables] -> device int32[n_samples+1]  */
    const int64_t *h_n_lookups;      /* host [n_tables]                               */
    /* 0 or 32: the indices are int32.  64: they are int64 (h_indices[z] then points at
     * device int64[n_lookups_z]); accepted by fae_profile and fae_partition_batch, whose
     * inputs are raw row ids; values outside [0, rows_z) are reported as FAE_ERANGE as
     * usual.  Hot sub-batches (hot slots) are always int32. */
    int32_t index_bits;
} fae_batch;

/* Where fae_build_hot_tables takes the weights of hot rows from. */
#define FAE_SRC_DEVICE 0     /* h_W[z] -> device fp32[rows_z * dim], materialised table     */
#define FAE_SRC_PROCEDURAL 1 /* virtual table: w(z,r,c) is a counter-based hash of seed     */
typedef struct {
    int32_t kind;
    const float *const *h_W; /* FAE_SRC_DEVICE only */
    uint64_t seed;           /* FAE_SRC_PROCEDURAL only */
} fae_weight_src;

/* Optional extra outputs of the backward for bit-exact checking: the distinct
 * hot slots touched per table in ascending order and their multiplicities,
 * concatenated table after table.  uniq/runlen need room for the total number of
 * lookups; table_start gets n_tables+1 entries (start of each table's part). */
typedef struct {
    int32_t *uniq;
    int32_t *runlen;
    int32_t *table_start;
} fae_bwd_debug;

/* ---- context -------------------------------------------------------------- */
/* Bind a context to a device and a HIP stream (hipStream_t passed as void*;
 * NULL = the default stream).  Allocates the two 4 KiB status blocks. */
int32_t fae_create(fae_ctx **out, int32_t device, void *hip_stream);
void fae_destroy(fae_ctx *ctx);
const char *fae_last_error(const fae_ctx *ctx);
const char *fae_version(void);
/* Wait for the stream; return and clear the deferred device status. */
int32_t fae_sync(fae_ctx *ctx);
/* Tuning/ablation switches, e.g. ("profile_variant", 0=auto 1=global atomics
 * 2=LDS-privatised), ("fwd_variant", 0=auto 1=group-per-bag 2=wave-per-bag),
 * ("sort_variant", 0=auto, 1=global radix with three kernels per pass, 2=LDS per table
 * where it fits, 3=global radix with one kernel per pass, 4=the same with tiles handed out
 * by a counter), ("sort_order", 0=the lookups of a slot stay in batch order, 1=the LDS sort
 * places lookups by counting: faster on small batches, but the order inside a slot's run, and
 * with it the last bits of the updated weights, may differ from run to run), ("reduce_variant", 0=auto
 * 1=segmented scan across lane groups 2=a share of the span per lane group),
 * ("reduce_span", 0/64/128/256 sorted lookups per wave), ("reduce_unroll", 0/4/8 gradient
 * rows in flight per lane group, second form only), ("reduce_wg_waves", 0=auto (1)/1/2/4
 * waves per workgroup of the reduce kernel), ("fixup_variant", 0=auto: runs that
 * cross the reduce kernel's spans are finished inside it, 1=by a kernel of their own),
 * ("fwd_stream_out", 0/1), ("handoff_fences", 0=the sums that one workgroup of the reduce kernel
 * hands to another are written and read with device-scope accesses and ordered by a wave-level
 * fence, 1=they are bracketed by device-scope release/acquire fences as well). */
int32_t fae_set_option(fae_ctx *ctx, const char *name, int64_t value);

/* ---- per-kernel timing (measurement aid; off by default) ---------------------- */
/* When enabled, every kernel launch of the library carries two HIP events that the
 * device stamps at the kernel's own start and end, so a figure holds the kernel and
 * nothing else (no host launch latency, whether or not the stream was idle).
 * fae_timing_read synchronises and returns, for one kernel class, the summed duration
 * and the number of launches since the last reset.  Keep it off while a stream of the
 * context is being captured into a graph: such launches cannot be captured. */
#define FAE_K_FWD 0          /* pooled forward                                  */
#define FAE_K_BWD_KEYS 1     /* (slot, sample) pairs                            */
#define FAE_K_SORT_HIST 2    /* radix pass: per-tile digit histogram            */
#define FAE_K_SORT_COLSCAN 3 /* radix pass: scan of digit counts over tiles     */
#define FAE_K_SORT_SCATTER 4 /* radix pass: stable scatter                      */
#define FAE_K_BWD_REDUCE 5   /* segment reduce + SGD                            */
#define FAE_K_BWD_FIXUP 6    /* runs that cross span boundaries: combine + SGD  */
#define FAE_K_LDS_SORT 7     /* per-table sort inside one workgroup's LDS       */
#define FAE_K_FILL 8         /* fills / clears                                  */
#define FAE_K_PROFILE 9      /* access histogram                                */
#define FAE_K_PARTITION 10   /* input classifier kernels                        */
#define FAE_K_BUILD 11       /* classify / scan / gather                        */
#define FAE_K_OTHER 12
#define FAE_K_COPY_PROBE 13  /* plain streaming copy (bandwidth ceiling, counter calibration) */
#define FAE_K_FWD_SORT 14    /* forward and the backward's LDS sort in one launch */
#define FAE_K_SYNC_ROWS 15   /* hot rows <-> full tables                          */
#define FAE_K_ESTIMATE 16    /* chunk counts of the sampled logger                */
#define FAE_K_READ_PROBE 17  /* plain streaming read (read-only bandwidth ceiling)      */
#define FAE_K_FILL_PROBE 18  /* plain streaming fill (write-only bandwidth ceiling)     */
#define FAE_K_COUNT 19
int32_t fae_timing_enable(fae_ctx *ctx, int32_t on);
int32_t fae_timing_reset(fae_ctx *ctx);
int32_t fae_timing_read(fae_ctx *ctx, int32_t kernel_class, double *h_total_ms, int64_t *h_launches);
const char *fae_kernel_name(int32_t kernel_class);
/* Plain device-to-device streaming copy of `bytes` (multiple of 16) by a 16-byte-per-lane
 * kernel: what a bandwidth-bound kernel can reach on this device, and a transfer of known
 * size against which hardware byte counters are scaled.  The three probes take their launch
 * shape from the options ("probe_unroll", 0=best known, 1/2/4/8 accesses in flight per lane),
 * ("probe_nt", -1=best known, 0/1 non-temporal accesses) and ("probe_wgs_per_cu", 0=one
 * workgroup of 256 lanes per chunk of unroll*256 vectors, n=n workgroups per compute unit
 * striding over the chunks).  Asynchronous. */
int32_t fae_copy_probe(fae_ctx *ctx, void *dst, const void *src, size_t bytes);
/* The same, writing only: `bytes` of dst are set to `value`. */
int32_t fae_fill_probe(fae_ctx *ctx, void *dst, size_t bytes, float value);
/* The same access pattern, reading only: `bytes` (multiple of 16) of src are loaded and
 * summed; nothing is stored unless the sum has one particular value, in which case one float
 * goes to sink[0] (so the loads cannot be dropped).  What a read-dominated kernel can reach
 * on this device.  Asynchronous. */
int32_t fae_read_probe(fae_ctx *ctx, const void *src, size_t bytes, float *sink);

/* ---- a1: Embedding Logger (Sec. 4.1.2) ------------------------------------- */
/* counts_z[r] += number of lookups of `chunk` into row r of table z.  The caller
 * zeroes the counters before the first chunk; calls accumulate.  Asynchronous. */
int32_t fae_profile(fae_ctx *ctx, const fae_tables *tables, const fae_batch *chunk,
                    uint32_t *const *h_counts /* host [n_tables] -> device uint32[rows_z] */);

/* ---- a2: hot cutoff (Eq. 1, Eq. 2; budget L of Sec. 4.1) ------------------- */
/* Budget mode.  Tables with rows_z*dim*4 < small_table_bytes are wholly hot
 * (cutoff 0).  Every other table uses H_z(c) = ceil(c * h_T[z] / t_denom) and a row
 * is hot iff count >= H_z: the paper's threshold t, a fraction of a table's accesses,
 * on the integer grid t = c / t_denom.  Finds the smallest integer c >= 0 whose hot
 * rows (small tables included) fit budget_bytes.  h_T[z] is the number of profiled
 * lookups into table z; t_denom = max_z h_T[z] makes one step of c one access for the
 * most-accessed table (for one-hot tables that is the number of profiled samples).  Outputs (host): *h_c_out, h_cutoff_out[z], h_n_hot_out[z].
 * Synchronises.  FAE_ENOSPC if the small tables alone exceed the budget. */
size_t fae_choose_cutoff_workspace_bytes(const fae_tables *tables);
int32_t fae_choose_cutoff(fae_ctx *ctx, const fae_tables *tables, const uint32_t *const *h_counts,
                          const int64_t *h_T, int64_t t_denom, int64_t budget_bytes,
                          int64_t small_table_bytes, int64_t *h_c_out, uint32_t *h_cutoff_out,
                          int64_t *h_n_hot_out, void *ws, size_t ws_bytes);
/* Explicit mode helper: number of rows with count >= h_cutoff[z].  Synchronises. */
int32_t fae_count_hot(fae_ctx *ctx, const fae_tables *tables, const uint32_t *const *h_counts,
                      const uint32_t *h_cutoff, int64_t *h_n_hot_out, void *ws, size_t ws_bytes);

/* ---- a3 + a4: Embedding Classifier and Replicator (Sec. 4.2, Sec. 4) ------- */
/* Tags every row hot (count >= h_cutoff[z]) or cold in one pass, gives hot rows
 * consecutive slots in ascending row order, and fills the hot tables:
 *   remap_z[r]   = slot of r, or -1 if cold          (device int32[rows_z])
 *   hot_ids_z[s] = row id held by slot s               (device int32[h_cap[z]])
 *   hotW_z[s][:] = weights of row hot_ids_z[s]         (device fp32[h_cap[z]*dim])
 * h_cap[z] is the capacity (in rows) of hot_ids_z/hotW_z; if a table has more hot
 * rows than capacity nothing is written past it and FAE_ENOSPC is returned.
 * h_n_hot_out[z] (host) receives the hot-row counts.  Synchronises. */
size_t fae_build_workspace_bytes(const fae_tables *tables);
int32_t fae_build_hot_tables(fae_ctx *ctx, const fae_tables *tables, const uint32_t *const *h_counts,
                             const uint32_t *h_cutoff, const fae_weight_src *src,
                             int32_t *const *h_remap, int32_t *const *h_hot_ids,
                             float *const *h_hotW, const int64_t *h_cap, int64_t *h_n_hot_out,
                             void *ws, size_t ws_bytes);

/* ---- a5: Input Classifier (Sec. 4.2) --------------------------------------- */
/* A sample is hot iff every lookup in every table hits a hot row.  Outputs:
 *   hot_samples  int32[n_samples]  ids of hot samples, ascending (first *h_n_hot_samples valid)
 *   cold_samples int32[n_samples]  ids of cold samples, ascending
 *   h_slots[z]    -> device int32[n_lookups_z]  hot slots of the hot samples' lookups, in order
 *   h_hoffsets[z] -> device int32[n_samples+1]  CSR offsets of the hot sub-batch
 *   h_n_hot_lookups[z] (host) = lookups of the hot sub-batch in table z
 * The hot sub-batch (h_slots, h_hoffsets, *h_n_hot_samples, h_n_hot_lookups) is a
 * fae_batch over the hot tables; consecutive slices of it are the hot mini-batches.
 * Synchronises. */
size_t fae_partition_workspace_bytes(const fae_tables *tables, int64_t n_samples);
int32_t fae_partition_batch(fae_ctx *ctx, const fae_tables *tables, const fae_batch *in,
                            const int32_t *const *h_remap, int32_t *hot_samples,
                            int32_t *cold_samples, int64_t *h_n_hot_samples,
                            int32_t *const *h_slots, int32_t *const *h_hoffsets,
                            int64_t *h_n_hot_lookups, void *ws, size_t ws_bytes);

/* ---- a6: hot mini-batch forward (Fig. 2; sum pooling) ---------------------- */
/* out[s*out_row_stride + z*dim + c] = sum over the lookups j of bag (s,z) of
 * hotW_z[slot_j][c]; repeated slots count with multiplicity; an empty bag gives
 * zeros.  hot_tables->h_rows[z] = n_hot_z; hot_batch->h_indices hold hot slots.
 * out_row_stride (in floats) >= n_tables*dim.  Asynchronous. */
int32_t fae_embbag_fwd(fae_ctx *ctx, const fae_tables *hot_tables, const float *const *h_hotW,
                       const fae_batch *hot_batch, float *out, int64_t out_row_stride);

/* ---- a7 + a8: backward and sparse SGD on the GPU (Sec. 2.2, Sec. 6.2) ------ */
/* Per table: sorts the lookups by hot slot (stable), sums the upstream gradient
 * rows gout[s*gout_row_stride + z*dim + :] of duplicate slots, and applies
 * hotW_z[slot][:] -= lr * G[slot][:] once per distinct slot; untouched rows are
 * not written.  dbg may be NULL.  Asynchronous. */
size_t fae_bwd_workspace_bytes(const fae_tables *hot_tables, int64_t n_samples,
                               const int64_t *h_n_lookups);
/* Optional: start the sort of the backward (steps that depend only on the batch, not on
 * the gradient) on the context's side stream, so that it overlaps whatever runs on the
 * main stream between this call and fae_embbag_bwd_sgd (the forward, the dense layers).
 * It starts after all work queued on the main stream so far.  A following
 * fae_embbag_bwd_sgd with the same batch and workspace waits for it and skips its own
 * sort; with another batch in that workspace it waits and sorts itself.  "The same batch" means
 * the same index buffer, offset buffer and number of lookups for every table and the same
 * number of samples; the contents of those buffers and of the workspace must stay untouched in
 * between.  Sorted pairs are remembered per workspace, for
 * up to four workspaces at a time (beyond that the oldest are forgotten and their backward
 * call sorts again), so the next batch can be sorted into a second workspace while this
 * batch's forward and backward still run.  Asynchronous. */
int32_t fae_embbag_bwd_presort(fae_ctx *ctx, const fae_tables *hot_tables, const fae_batch *hot_batch,
                               void *ws, size_t ws_bytes);
/* fae_embbag_fwd that also carries the sort of the backward for the same batch: when every
 * table is one-hot and the batch is small enough for the in-LDS sort (<= 16384 samples),
 * one launch holds both, the sorting workgroups running beside the row copies; the sorted
 * pairs stay in ws for the fae_embbag_bwd_sgd call with the same batch and workspace.
 * For any other shape it is exactly fae_embbag_fwd.  Same results as the separate calls.
 * Asynchronous. */
int32_t fae_embbag_fwd_presort(fae_ctx *ctx, const fae_tables *hot_tables, const float *const *h_hotW,
                               const fae_batch *hot_batch, float *out, int64_t out_row_stride, void *ws,
                               size_t ws_bytes);
int32_t fae_embbag_bwd_sgd(fae_ctx *ctx, const fae_tables *hot_tables, float *const *h_hotW,
                           const fae_batch *hot_batch, const float *gout, int64_t gout_row_stride,
                           float lr, const fae_bwd_debug *dbg, void *ws, size_t ws_bytes);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): fae_embbag_bwd_sgd with the workspace inside the
 * library instead of the caller's.  The workspace is one array of FAE_BWD_STATIC_WS_BYTES per
 * device, part of the library's code object (every device the library runs on holds it until the
 * process ends); the call allocates and frees nothing.  Same arguments, results and error
 * behaviour as fae_embbag_bwd_sgd without the optional outputs; a batch whose
 * fae_bwd_workspace_bytes() exceeds FAE_BWD_STATIC_WS_BYTES is rejected with FAE_ENOSPC before
 * anything is launched (the need is about 32 bytes per lookup at dim 64, so about 1 M lookups
 * fit; fae_bwd_static_workspace_bytes() returns the limit).  Every call on a device uses that device's one array, which keeps the last call's
 * contents (the call clears what must start at zero): calls that overlap on one device, from
 * several contexts or streams, race; calls on one stream are ordered.  Asynchronous. */
#define FAE_BWD_STATIC_WS_BYTES (32u << 20)
size_t fae_bwd_static_workspace_bytes(void);
int32_t fae_embbag_bwd_sgd_static(fae_ctx *ctx, const fae_tables *hot_tables, float *const *h_hotW,
                                  const fae_batch *hot_batch, const float *gout, int64_t gout_row_stride,
                                  float lr);

/* ---- pooling and optimizer variants ----------------------------------------------
 * The paper names the pooled embedding lookup and the optimizer step (Sec. 2.2) without
 * fixing either; fae_embbag_fwd / fae_embbag_bwd_sgd are sum pooling and plain SGD.  These
 * entry points add the two other choices common in recommender training:
 *   FAE_POOL_MEAN   out = (sum of the bag's rows) / (lookups in the bag); an empty bag gives
 *                   zeros; in the backward every lookup receives its bag's gradient / length.
 *   FAE_OPT_ROWWISE_ADAGRAD   one fp32 accumulator per hot row (h_state[z] -> device
 *                   fp32[n_hot_z], zero before the first step).  Per distinct row of a step,
 *                   with G the summed gradient of the row:
 *                     acc += (1/dim) * sum_c G[c]^2;  w[c] -= lr * G[c] / (sqrt(acc) + eps).
 *                   Needs dim <= 256 (dim <= 64 when dim % 4 != 0).
 * With FAE_POOL_SUM and FAE_OPT_SGD they are the plain calls.  Asynchronous. */
#define FAE_POOL_SUM 0
#define FAE_POOL_MEAN 1
#define FAE_OPT_SGD 0
#define FAE_OPT_ROWWISE_ADAGRAD 1
typedef struct {
    int32_t pooling;
    int32_t optimizer;
    float lr;
    float eps;             /* FAE_OPT_ROWWISE_ADAGRAD only */
    float *const *h_state; /* FAE_OPT_ROWWISE_ADAGRAD only */
} fae_step_opts;
int32_t fae_embbag_fwd_opts(fae_ctx *ctx, const fae_tables *hot_tables, const float *const *h_hotW,
                            const fae_batch *hot_batch, float *out, int64_t out_row_stride,
                            const fae_step_opts *opts);
int32_t fae_embbag_bwd_opts(fae_ctx *ctx, const fae_tables *hot_tables, float *const *h_hotW,
                            const fae_batch *hot_batch, const float *gout, int64_t gout_row_stride,
                            const fae_step_opts *opts, const fae_bwd_debug *dbg, void *ws, size_t ws_bytes);

/* ---- embedding synchronisation between the hot tables and the full tables ----
 * (Sec. 3 (4); Sec. 6.2, "Embedding Synchronization") */
/* When training switches between hot and cold mini-batches the two copies of the hot
 * rows are brought in line:
 *   FAE_SYNC_HOT_TO_FULL  W_z[hot_ids_z[s]][:] = hotW_z[s][:]   (before cold mini-batches)
 *   FAE_SYNC_FULL_TO_HOT  hotW_z[s][:] = W_z[hot_ids_z[s]][:]   (before hot mini-batches)
 * for s in [0, h_n_hot[z]).  tables describes the full tables (rows_z, dim); h_W[z] is
 * fp32[rows_z*dim] in memory the device can address (device memory, or pinned host
 * memory mapped into the device's address space, in which case the host link sets the
 * rate).  Rows of the destination that are not named stay untouched.  hot_ids_z must not
 * repeat a row (fae_build_hot_tables never does); an id outside [0, rows_z) is skipped
 * and reported as FAE_ERANGE by the next synchronising call.  Asynchronous. */
#define FAE_SYNC_HOT_TO_FULL 0
#define FAE_SYNC_FULL_TO_HOT 1
int32_t fae_sync_hot_rows(fae_ctx *ctx, const fae_tables *tables, const int64_t *h_n_hot,
                          const int32_t *const *h_hot_ids, float *const *h_hotW,
                          float *const *h_W, int32_t direction);

/* ---- hot-size estimate from sampled chunks of the logger (Sec. 4.1.2, Eq. 2-4) ---- */
/* The logger of table z is cut into N_z = ceil(rows_z / m) aligned chunks of m entries
 * (the last one may be short).  The caller draws h_n_chunks[z] distinct chunk numbers
 * per table (the paper: n = 35 chunks of m = 1024 entries) and passes them in
 * h_chunks[z] (host int64[h_n_chunks[z]]); the library draws no random numbers.
 *   C_i   = entries of chunk i with count >= h_cutoff[z]                       (Eq. 2)
 *   ybar  = mean of the C_i, s = their sample standard deviation (n - 1)       (Eq. 3)
 *   half  = t_{alpha/2, n-1} * sqrt(((N - n) / N) * s^2 / n), alpha = 1 - confidence  (Eq. 4)
 * and, scaled to the table, rows = ybar * N_z and half_rows = half * N_z.  A table with a
 * single sampled chunk has no standard deviation: s and half are reported as 0.
 * The counting runs on the device (one workgroup per chunk); the statistics of the at
 * most FAE_MAX_TABLES * n counts are taken on the host in fp64.  h_C_out (optional, host
 * int32, table after table, h_n_chunks[z] entries each) receives the C_i.  Synchronises. */
typedef struct {
    double rows;      /* estimated number of hot rows of the table: ybar * N */
    double half_rows; /* half-width of its confidence interval, in rows      */
    double ybar;      /* Eq. 3                                               */
    double s;         /* sample standard deviation of the chunk counts       */
    int64_t N;        /* chunks in the table                                 */
    int64_t n;        /* chunks sampled                                      */
} fae_hot_estimate;
size_t fae_estimate_workspace_bytes(const fae_tables *tables, const int64_t *h_n_chunks);
int32_t fae_estimate_hot(fae_ctx *ctx, const fae_tables *tables, const uint32_t *const *h_counts,
                         const uint32_t *h_cutoff, int64_t m, const int64_t *h_n_chunks,
                         const int64_t *const *h_chunks, double confidence,
                         fae_hot_estimate *h_out /* host [n_tables] */, int32_t *h_C_out,
                         void *ws, size_t ws_bytes);
/* Statistical Optimizer (Sec. 4.1.2, "Converging on a Threshold") on the sampled logger:
 * fae_choose_cutoff with the exact row counts replaced by the estimates above.  Finds the
 * smallest integer c >= 0 with  sum_z bytes_z(c) <= budget_bytes, where for a table below
 * small_table_bytes bytes_z = rows_z*dim*4 (wholly hot, not sampled) and otherwise
 * bytes_z(c) = (sumC_z(c) / n_z) * N_z * (dim*4) in fp64, summed in table order, with
 * H_z(c) = ceil(c * h_T[z] / t_denom).  The same chunks serve every c, so the estimate
 * falls monotonically in c and a bisection finds the answer.  h_out receives the estimates
 * at the chosen c (interval at `confidence`).  Synchronises. */
int32_t fae_choose_cutoff_sampled(fae_ctx *ctx, const fae_tables *tables, const uint32_t *const *h_counts,
                                  const int64_t *h_T, int64_t t_denom, int64_t budget_bytes,
                                  int64_t small_table_bytes, int64_t m, const int64_t *h_n_chunks,
                                  const int64_t *const *h_chunks, double confidence, int64_t *h_c_out,
                                  uint32_t *h_cutoff_out, fae_hot_estimate *h_out, void *ws,
                                  size_t ws_bytes);
/* Quantile t_{alpha/2} of Student's t distribution with df degrees of freedom for a
 * two-sided interval of the given confidence (0 < confidence < 1, df >= 1).  Host only. */
double fae_t_quantile(double confidence, int64_t df);

/* ---- Shuffle Scheduler rate rule (Sec. 5, Eq. 5); host only ------------------- */
/* The rate R(p), p in [1, 100]: p per cent of the cold (then of the hot) mini-batches
 * run between two swaps.  After every swap the caller reports the test loss:
 *   loss >= previous loss                      -> p = max(p / 2, 1)
 *   loss fell at each of the last u reports    -> p = min(2 p, 100), count starts again
 *   otherwise                                  -> p unchanged
 * (the clamps follow the text of Sec. 5: never below R(1), never above R(100)).
 * fae_sched_init sets p = p0 (the paper starts at R(50)) and u (the paper: 4). */
typedef struct {
    double rate;     /* p of R(p)                                 */
    double prev;     /* loss of the previous report               */
    int32_t u;       /* successive falls that double the rate     */
    int32_t falls;   /* successive falls seen since the last change */
    int32_t reports; /* losses reported so far                    */
} fae_sched;
int32_t fae_sched_init(fae_sched *s, double p0, int32_t u);
/* Returns the rate after taking this loss into account (negative on a bad argument). */
double fae_sched_report(fae_sched *s, double test_loss);
/* Mini-batches to run before the next swap at the current rate, out of n_total of that
 * kind: ceil(p / 100 * n_total), at least 1 (0 if n_total is 0). */
int64_t fae_sched_segment(const fae_sched *s, int64_t n_total);

#ifdef __cplusplus
}
#endif
#endif /* FAE_H */
