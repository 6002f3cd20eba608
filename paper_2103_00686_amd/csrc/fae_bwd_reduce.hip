// Backward, steps 3 + 4: segment reduce of the sorted lookups and the optimizer step on the hot
// tables (Sec. 2.2, Sec. 6.2).  One wave owns a span of sorted lookups; runs inside the span get
// their update at once, runs that cross span borders are finished by the span in which they end
// (or by the fix-up kernel).  No float atomics: every row has one writer, and the sums are added
// in the order the sort stage delivers the lookups.  Also here: the optional outputs for bit-exact checking (distinct slots, multiplicities).
#include "fae_bwd.h"

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

__device__ __forceinline__ SpanInfo bwd_span_info(const BwdArgs &a, int sid, int z)
{
    SpanInfo s;
    s.z = z;
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

// Runs that cross span borders are finished by the span in which they end: it adds the pieces
// the earlier spans have published (their tail sum where the run began, their whole-span sums in
// between) to its own head sum and applies the update.  It only ever waits for spans with smaller
// numbers, which the hardware starts first (workgroups are dispatched in the order of their
// numbers; fixup_variant=1 finishes these runs in a kernel of its own and needs no such order);
// the wait is bounded all the same, and a wave whose wait gives up sets the status word and
// leaves the row alone.  Called by every wave once its own border sums have been stored with
// bwd_store_shared.
//
// How the border sums reach the other workgroup (a.handoff):
//   0  every word of a border sum is stored, and later loaded, with a device-scope access (it
//      goes past the caches that belong to one part of the chip); the publishing wave waits
//      for its stores to be acknowledged (a wave-level release fence: all outstanding memory
//      operations of the wave, and no reordering by the compiler) and only then raises its flag;
//      the reader loads the sums only after it has seen the flag.
//   1  the same accesses, bracketed by device-scope fences as the memory model spells it out:
//      release (write back this part's cache) before the flag is raised, acquire (drop this
//      part's cached copies) after it has been seen.  On a chip whose second-level caches are
//      per part these fences work on the whole cache, not on the few rows that matter.
template <typename V, int LPR>
__device__ __forceinline__ void bwd_finish_borders(const BwdArgs &a, const SpanInfo &sp, int sid, int n_hot, V *W,
                                                   V *part, int ncols)
{
    constexpr int G = FAE_WAVE / LPR;
    const int lane = fae_lane(), g = lane / LPR, l = lane % LPR;
    const int c = l; // one column slice per lane: the host takes this path only when the row fits LPR lanes
    const bool active = c < ncols;
    if (sp.head_open || sp.tail_open) {
        if (a.handoff == 1)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        else
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0): every lane's border sums have been acknowledged
        __builtin_amdgcn_wave_barrier();
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
    bool gave_up = false;
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
                gave_up = true;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        if (gave_up)
            break;
        if (a.handoff == 1)
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        else
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
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
    // a wait that gave up in any lane group: the row (and its accumulator) stays as it was; the
    // status word makes the next synchronising call report the step as invalid
    if (__ballot(gave_up) != 0)
        return;
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

// One batch of the reduce kernel's main loop: UN steps of G gradient rows each, and whatever
// else those steps read (the weight row of a run that ends there, its Adagrad accumulator).
template <typename V, int UN, bool VAR> struct BwdBatch {
    int kk[UN], dd[UN];
    V vv[UN], ww[UN];
    float inv[VAR ? UN : 1], sw[VAR ? UN : 1];
};

// UN = steps per batch; the loads of a batch are issued before the batch in front of it is summed
// (two batches alternate), so a wave always has rows on their way while it works.  VAR = mean
// pooling or Adagrad may be asked for (the plain kernel carries neither their registers nor
// their branches).
template <typename V, int LPR, int UNMAX, bool VAR> __global__ __launch_bounds__(256) void bwd_reduce_kernel(BwdArgs a)
{
    constexpr int G = FAE_WAVE / LPR;              // lane groups = gradient rows per step
    constexpr int VW = sizeof(V) / sizeof(float);
    constexpr int STEPS = FAE_WAVE / G;            // steps per tile of 64 lookups
    constexpr int UN = STEPS < UNMAX ? STEPS : UNMAX; // steps whose loads are issued together
    constexpr int NBATCH = STEPS / UN;
    typedef BwdBatch<V, UN, VAR> Batch;
    // the same for every lane of a wave: said so, the span's bookkeeping runs on the scalar unit
    const int sid = blockIdx.x * a.wg_waves + __builtin_amdgcn_readfirstlane(threadIdx.x / FAE_WAVE);
    // the table is looked up before the range check: kernel arguments only, so these loads leave
    // together with the first ones instead of after them
    const int z_of_span = fae_find_table(a.blk_start, a.n_tables, sid);
    if (sid >= a.n_spans)
        return;
    const int lane = fae_lane(), g = lane / LPR, l = lane % LPR;
    // The span's place follows from the kernel arguments alone, so the pairs of its first 64
    // lookups are asked for in the same round as the status word and the span's border keys.
    int knext_tile, snext_tile;
    {
        const int seg0 = a.seg_start[z_of_span], seg1 = a.seg_start[z_of_span + 1];
        const int pos0 = seg0 + (sid - a.blk_start[z_of_span]) * a.span;
        const int pos1 = pos0 + a.span < seg1 ? pos0 + a.span : seg1;
        const int p = pos0 + lane;
        knext_tile = p < pos1 ? a.keys_in[p] : KEY_NONE;
        snext_tile = p < pos1 ? a.vals_in[p] : 0;
    }
    // a bounded wait of the sort stage gave up: the pairs are not what they should be
    const uint32_t status = __hip_atomic_load(a.status + FAE_BLK_STATUS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const SpanInfo sp = bwd_span_info(a, sid, z_of_span);
    if (status & FAE_STATUS_EINTERNAL)
        return;
    const int ncols = a.dim / VW;
    const int n_hot = a.n_hot[sp.z];
    V *W = (V *)a.W[sp.z];
    const float *gbase = a.gout + (int64_t)sp.z * a.dim;
    V *part = (V *)(a.partial + (int64_t)sid * 2 * a.dim);
    const bool mean = VAR && a.mean, adagrad = VAR && a.adagrad;

    for (int c0 = 0; c0 < ncols; c0 += LPR) {
        const int c = c0 + l;
        const bool active = c < ncols;
        // Sum of the run that is open at the end of the previous step.  It lives in the last lane
        // group only: the rotations of the scan below hand it to the groups that continue the run.
        V cv = bwd_vec<V>::zero();
        int klast = KEY_NONE; // last key of the previous tile (none at the span's start)
        int dist_in = 0;      // position inside its run of a lookup that continues the previous tile's last run
        if (c0 > 0) { // rows wider than one pass over the lanes: the first tile's pairs again
            const int p = sp.pos0 + lane;
            knext_tile = p < sp.pos1 ? a.keys_in[p] : KEY_NONE;
            snext_tile = p < sp.pos1 ? a.vals_in[p] : 0;
        }
        for (int t0 = sp.pos0; t0 < sp.pos1; t0 += FAE_WAVE) {
            const int p = t0 + lane;
            const int kreg = knext_tile;
            const int sreg = snext_tile;
            // key that follows each lookup; the span's last lookup always closes its run here
            int kafter = __shfl_down(kreg, 1, FAE_WAVE);
            if (lane == FAE_WAVE - 1)
                kafter = t0 + FAE_WAVE < sp.pos1 ? a.keys_in[t0 + FAE_WAVE] : KEY_NONE;
            if (p == sp.pos1 - 1)
                kafter = KEY_NONE;
            { // the pairs of the next tile: asked for now, used after this tile's rows
                const int pn = p + FAE_WAVE;
                knext_tile = pn < sp.pos1 ? a.keys_in[pn] : KEY_NONE;
                snext_tile = pn < sp.pos1 ? a.vals_in[pn] : 0;
            }
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
            if (mean && a.offsets[sp.z] && p < sp.pos1) {
                const int32_t *off = a.offsets[sp.z];
                const int len = off[sreg + 1] - off[sreg];
                ireg = 1.0f / (float)(len > 0 ? len : 1);
            }
            klast = __builtin_amdgcn_readlane(kreg, FAE_WAVE - 1);
            dist_in = __builtin_amdgcn_readlane(dist, FAE_WAVE - 1) + 1;

            // every load of a batch is issued before the first use of any of them
            auto issue = [&](Batch &b, int i0) {
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int e = (i0 + u) * G + g;
                    b.kk[u] = __shfl(kreg, e, FAE_WAVE);
                    b.dd[u] = __shfl(dreg, e, FAE_WAVE);
                    const int s = __shfl(sreg, e, FAE_WAVE);
                    if (VAR)
                        b.inv[u] = mean ? __shfl(ireg, e, FAE_WAVE) : 1.0f;
                    b.vv[u] = (active && b.kk[u] != KEY_NONE) ? ((const V *)(gbase + (int64_t)s * a.gout_stride))[c]
                                                             : bwd_vec<V>::zero();
                    b.ww[u] = (active && (b.dd[u] & 3) == 1) ? W[(int64_t)b.kk[u] * ncols + c] : bwd_vec<V>::zero();
                    if (VAR)
                        b.sw[u] = (adagrad && (b.dd[u] & 3) == 1) ? a.opt_state[sp.z][b.kk[u]] : 0.f;
                }
            };
            auto sum = [&](Batch &b) {
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int kg = b.kk[u];
                    const int dest = b.dd[u] & 3, dist_u = b.dd[u] >> 2;
                    V vg = b.vv[u];
                    if (mean)
                        bwd_vec<V>::scale(vg, b.inv[u]);
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
                    if (adagrad) { // one accumulator per row: grows by the row's mean squared gradient
                        float q = bwd_vec<V>::sumsq(vg);
#pragma unroll
                        for (int m = 1; m < LPR; m <<= 1)
                            q += __shfl_xor(q, m, FAE_WAVE);
                        const float acc = b.sw[u] + q / (float)a.dim;
                        step = a.lr / (sqrtf(acc) + a.eps);
                        if (dest == 1 && l == 0)
                            a.opt_state[sp.z][kg] = acc;
                    }
                    if (active) {
                        if (dest == 1)
                            W[(int64_t)kg * ncols + c] = bwd_vec<V>::sgd(b.ww[u], vg, step);
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
            };
            // batches past the span's end hold nothing: they are neither asked for nor summed
            const int n_batch = (sp.pos1 - t0 >= FAE_WAVE) ? NBATCH : ((sp.pos1 - t0) + UN * G - 1) / (UN * G);
            Batch b0, b1;
            issue(b0, 0);
#pragma unroll
            for (int ib = 0; ib < NBATCH; ib += 2) {
                if (ib >= n_batch)
                    break;
                if (ib + 1 < NBATCH && ib + 1 < n_batch)
                    issue(b1, (ib + 1) * UN);
                sum(b0);
                if (ib + 1 < NBATCH && ib + 1 < n_batch) {
                    if (ib + 2 < NBATCH && ib + 2 < n_batch)
                        issue(b0, (ib + 2) * UN);
                    sum(b1);
                }
            }
        }
    }
    if (a.fused_fixup)
        bwd_finish_borders<V, LPR>(a, sp, sid, n_hot, W, part, ncols);
}

// Segment reduce + SGD, second form: no traffic between lanes while the gradient rows are
// summed, and as few instructions per gradient row as it takes.  A wave still owns a span of
// sorted lookups, but each of its 64/LPR lane groups walks its own contiguous share of the span,
// NB gradient rows in flight per group and a running sum per run (kept with selects).  The wave
// copies the (slot, sample) pairs of its span into LDS once (coalesced) and each group reads the
// pairs of its share from there four at a time (one address per group, a broadcast), so the shape
// of the runs is known when a batch's loads are issued: the weight row of every run that closes
// strictly inside the share is loaded together with the gradient rows and updated as soon as the
// run's sum is complete.  Rows are addressed with a 32-bit byte offset from the table's or the
// gradient's base (the host takes this form only where every offset fits: see bwd_walk_fits).
// What is left per group is its first and its last run; one pass over the groups, in order,
// joins those that continue each other and sends every joined run to its place: the weight row
// (fetched ahead by the group in which the run ends), or the span's head / tail scratch row when
// the run crosses the span's border.  Plain SGD on summed rows of float4 columns that fit one
// pass over the lanes of a group; everything else runs in the first form.
template <int LPR, int NB> __global__ __launch_bounds__(256) void bwd_reduce_walk_kernel(BwdArgs a)
{
    typedef float4 V;
    constexpr int G = FAE_WAVE / LPR;
    __shared__ __align__(16) int lk[256 / FAE_WAVE][BWD_SPAN_MAX + 4];
    __shared__ __align__(16) int lv[256 / FAE_WAVE][BWD_SPAN_MAX];
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / FAE_WAVE);
    const int sid = blockIdx.x * a.wg_waves + wv;
    // the table is looked up before the range check: kernel arguments only, so these loads leave
    // together with the first ones instead of after them
    const int z_of_span = fae_find_table(a.blk_start, a.n_tables, sid);
    if (sid >= a.n_spans)
        return;
    // a bounded wait of the sort stage gave up: the pairs are not what they should be
    const uint32_t status = __hip_atomic_load(a.status + FAE_BLK_STATUS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const SpanInfo sp = bwd_span_info(a, sid, z_of_span);
    if (status & FAE_STATUS_EINTERNAL)
        return;
    const int lane = fae_lane(), g = lane / LPR, l = lane % LPR;
    const int ncols = a.dim / 4;
    const int n_hot = a.n_hot[sp.z];
    V *W = (V *)a.W[sp.z];
    const char *wb = (const char *)W;
    const char *gb = (const char *)(a.gout + (int64_t)sp.z * a.dim);
    V *part = (V *)(a.partial + (int64_t)sid * 2 * a.dim);
    const int share = a.span / G; // lookups per group: a multiple of NB (the span is a multiple of 64)
    const bool active = l < ncols;
    const uint32_t colb = (uint32_t)l * sizeof(V);
    const uint32_t rowb = (uint32_t)a.dim * sizeof(float);
    const uint32_t gstrideb = (uint32_t)a.gout_stride * sizeof(float);

    // the span's pairs; past its end a key that matches no slot and sample 0 (a row that exists)
    {
        constexpr int T = BWD_SPAN_MAX / FAE_WAVE;
        int fk[T], fv[T];
#pragma unroll
        for (int t = 0; t < T; ++t) { // every load is issued before the first store (indices clamped into the span)
            const int p = sp.pos0 + t * FAE_WAVE + lane;
            const int pc = p < sp.pos1 ? p : sp.pos1 - 1;
            fk[t] = a.keys_in[pc];
            fv[t] = a.vals_in[pc];
        }
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int i = t * FAE_WAVE + lane;
            const bool in = sp.pos0 + i < sp.pos1;
            if (i < a.span) {
                lk[wv][i] = in ? fk[t] : KEY_NONE;
                lv[wv][i] = in ? fv[t] : 0;
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int *mk = lk[wv] + g * share;
    const int *mv = lv[wv] + g * share;

    // Weight rows of the share's first and last run, for whichever joined run ends there (the pass
    // over the groups below).  Their slots are the share's first and last key; no lane of the
    // launch writes these rows before that pass, so they can be fetched ahead of everything else.
    V wh = bwd_vec<V>::zero(), wt = bwd_vec<V>::zero();
    if (active) {
        const int k0 = mk[0], k1 = mk[share - 1];
        if (k0 < n_hot)
            wh = *(const V *)(wb + (__umul24((uint32_t)k0, rowb) + colb));
        if (k1 < n_hot)
            wt = *(const V *)(wb + (__umul24((uint32_t)k1, rowb) + colb));
    }
    int cur = KEY_NONE; // key of the run being summed
    V acc = bwd_vec<V>::zero();
    int hk = KEY_NONE;  // the share's first run, once it has closed inside the share
    V hv = bwd_vec<V>::zero();
    bool multi = false;       // a run has closed inside the share
    bool multi_ahead = false; // the same, as of the batch whose loads are being issued
    if (active) {
        for (int j = 0; j < share; j += NB) {
            int kk[NB + 1], ss[NB];
#pragma unroll
            for (int u = 0; u < NB; u += 4) {
                const int4 k4 = *(const int4 *)(mk + j + u);
                const int4 s4 = *(const int4 *)(mv + j + u);
                kk[u] = k4.x; kk[u + 1] = k4.y; kk[u + 2] = k4.z; kk[u + 3] = k4.w;
                ss[u] = s4.x; ss[u + 1] = s4.y; ss[u + 2] = s4.z; ss[u + 3] = s4.w;
            }
            // the share's last lookup never closes its run here: the pass over the groups below does
            kk[NB] = j + NB < share ? mk[j + NB] : kk[NB - 1];
            V vv[NB], ww[NB];
            bool closes[NB];
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                vv[u] = *(const V *)(gb + (__umul24((uint32_t)ss[u], gstrideb) + colb));
                closes[u] = kk[u + 1] != kk[u];
                if (closes[u] && multi_ahead && kk[u] < n_hot) // read under the same condition below
                    ww[u] = *(const V *)(wb + (__umul24((uint32_t)kk[u], rowb) + colb));
                multi_ahead = multi_ahead || closes[u];
            }
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const bool same = kk[u] == cur;
                acc.x = (same ? acc.x : 0.f) + vv[u].x;
                acc.y = (same ? acc.y : 0.f) + vv[u].y;
                acc.z = (same ? acc.z : 0.f) + vv[u].z;
                acc.w = (same ? acc.w : 0.f) + vv[u].w;
                cur = kk[u];
                if (closes[u]) {
                    if (!multi) {
                        hk = cur;
                        hv = acc;
                    } else if (cur < n_hot) {
                        *(V *)(const_cast<char *>(wb) + (__umul24((uint32_t)cur, rowb) + colb)) =
                            bwd_vec<V>::sgd(ww[u], acc, a.lr);
                    }
                    multi = true;
                }
            }
        }
    }
    // a joined run with key k and sum v that ends in group `at` (as its first run if head)
    const int c = l;
    auto flush = [&](int at, bool head, int k, const V &v) {
        if (g != at || !active || k >= n_hot)
            return;
        if (sp.head_open && k == sp.first_key) {
            if (a.fused_fixup)
                bwd_store_shared(&part[c], v);
            else
                part[c] = v;
        } else if (sp.tail_open && k == sp.last_key) {
            if (a.fused_fixup)
                bwd_store_shared(&part[ncols + c], v);
            else
                part[ncols + c] = v;
        } else {
            W[(int64_t)k * ncols + c] = bwd_vec<V>::sgd(head ? wh : wt, v, a.lr);
        }
    };
    int ck = KEY_NONE, gprev = 0;
    V cv = bwd_vec<V>::zero();
#pragma unroll
    for (int gp = 0; gp < G; ++gp) {
        const int e_tk = __builtin_amdgcn_readlane(cur, gp * LPR);
        const int e_multi = __builtin_amdgcn_readlane((int)multi, gp * LPR);
        if (e_tk == KEY_NONE && !e_multi)
            continue; // a share that lies past the span's end
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
            ck = e_tk; // no key (the span ends inside this share): nothing is carried on
            cv = e_tv;
        } else {
            ck = fk;
            cv = first;
        }
        gprev = gp;
    }
    if (ck != KEY_NONE)
        flush(gprev, false, ck, cv);
    if (a.fused_fixup)
        bwd_finish_borders<V, LPR>(a, sp, sid, n_hot, W, part, ncols);
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
    const SpanInfo sp = bwd_span_info(a, sid, fae_find_table(a.blk_start, a.n_tables, sid));
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
// the second form exists for float4 columns on 4 to 64 lanes per row (the host asks for no other)
template <typename V, int LPR> void launch_walk(fae_ctx *ctx, const BwdArgs &a, dim3 grid, dim3 block)
{
    if constexpr (sizeof(V) == sizeof(float4) && LPR >= 4) {
        if (ctx->opt_unroll != 4 && a.span / (FAE_WAVE / LPR) >= 8)
            FAE_LAUNCH(ctx, (bwd_reduce_walk_kernel<LPR, 8>), grid, block, 0, ctx->stream, a);
        else
            FAE_LAUNCH(ctx, (bwd_reduce_walk_kernel<LPR, 4>), grid, block, 0, ctx->stream, a);
    }
}

template <typename V, int LPR> void launch_reduce(fae_ctx *ctx, const BwdArgs &a)
{
    {
        fae_ktimer kt(ctx, FAE_K_BWD_REDUCE);
        const dim3 grid((a.n_spans + a.wg_waves - 1) / a.wg_waves), block(a.wg_waves * FAE_WAVE);
        if (a.form == 1)
            launch_walk<V, LPR>(ctx, a, grid, block);
        else
        {
            // steps per batch: two where a step moves whole rows with few lanes to spare (long rows),
            // four otherwise; reduce_unroll 2 / 4 forces one
            const bool var = a.mean || a.adagrad;
            const int un = ctx->opt_unroll == 2 ? 2 : (ctx->opt_unroll == 4 ? 4 : 2);
            if (var)
                FAE_LAUNCH(ctx, (bwd_reduce_kernel<V, LPR, 2, true>), grid, block, 0, ctx->stream, a);
            else if (un == 2)
                FAE_LAUNCH(ctx, (bwd_reduce_kernel<V, LPR, 2, false>), grid, block, 0, ctx->stream, a);
            else
                FAE_LAUNCH(ctx, (bwd_reduce_kernel<V, LPR, 4, false>), grid, block, 0, ctx->stream, a);
        }
    }
    if (a.fused_fixup)
        return;
    fae_ktimer kt(ctx, FAE_K_BWD_FIXUP);
    FAE_LAUNCH(ctx, (bwd_fixup_kernel<V, LPR>), dim3((a.n_spans + 3) / 4), dim3(256), 0, ctx->stream, a);
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

void bwd_launch_reduce(fae_ctx *ctx, const BwdArgs &a, bool vec, int lpr)
{
#define CALL_REDUCE(V, L) launch_reduce<V, L>(ctx, a)
    if (vec) {
        BWD_LPR_SWITCH(float4, lpr, CALL_REDUCE)
    } else {
        BWD_LPR_SWITCH(float, lpr, CALL_REDUCE)
    }
#undef CALL_REDUCE
}

int32_t bwd_launch_debug(fae_ctx *ctx, BwdArgs &a)
{
    const int64_t N = a.seg_start[a.n_tables];
    FAE_LAUNCH(ctx, dbg_count_kernel, dim3((unsigned)a.dbg_tiles), dim3(256), 0, ctx->stream, a);
    FAE_LAUNCH_CHECK(ctx);
    int32_t rc = fae_scan_i32(ctx, a.dbg_tile_sums, a.dbg_tiles);
    if (rc != FAE_OK)
        return rc;
    FAE_LAUNCH(ctx, dbg_emit_kernel, dim3((unsigned)a.dbg_tiles), dim3(256), 0, ctx->stream, a);
    FAE_LAUNCH_CHECK(ctx);
    int rl_blocks = (int)((N + 255) / 256);
    if (rl_blocks > 4096)
        rl_blocks = 4096;
    FAE_LAUNCH(ctx, dbg_runlen_kernel, dim3(rl_blocks), dim3(256), 0, ctx->stream, a);
    FAE_LAUNCH_CHECK(ctx);
    return FAE_OK;
}
