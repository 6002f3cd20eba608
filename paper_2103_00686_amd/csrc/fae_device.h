// Device code shared by more than one kernel of libfae (gfx950).
#pragma once

#include "fae_internal.h"

#define RADIX_BITS 8
#define RADIX (1 << RADIX_BITS)
#define KEY_NONE 0x7fffffff // no carried run / element past the end of the span

// ---------------------------------------------------------------------------------
// 16-byte (or scalar) column slices
// ---------------------------------------------------------------------------------
template <typename V> struct vec_ops;
// s += v with the rounding error of the addition carried in c (compensated summation): the error
// of a long sum then stays at a few units of the last place whatever its length, also where one
// row is added over and over (a popular row in a long bag), which otherwise drifts one way.
__device__ __forceinline__ void fae_add_comp(float &s, float &c, float v)
{
    const float y = v - c;
    const float t = s + y;
    c = (t - s) - y;
    s = t;
}

template <> struct vec_ops<float4> {
    static __device__ __forceinline__ float4 zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ __forceinline__ void add(float4 &a, const float4 &b)
    {
        a.x += b.x;
        a.y += b.y;
        a.z += b.z;
        a.w += b.w;
    }
    static __device__ __forceinline__ void scale(float4 &a, float f)
    {
        a.x *= f;
        a.y *= f;
        a.z *= f;
        a.w *= f;
    }
    static __device__ __forceinline__ void add_comp(float4 &s, float4 &c, const float4 &v)
    {
        fae_add_comp(s.x, c.x, v.x);
        fae_add_comp(s.y, c.y, v.y);
        fae_add_comp(s.z, c.z, v.z);
        fae_add_comp(s.w, c.w, v.w);
    }
    static __device__ __forceinline__ float4 shfl_xor(const float4 &a, int m)
    {
        return make_float4(__shfl_xor(a.x, m, FAE_WAVE), __shfl_xor(a.y, m, FAE_WAVE),
                           __shfl_xor(a.z, m, FAE_WAVE), __shfl_xor(a.w, m, FAE_WAVE));
    }
};
template <> struct vec_ops<float> {
    static __device__ __forceinline__ float zero() { return 0.f; }
    static __device__ __forceinline__ void add(float &a, const float &b) { a += b; }
    static __device__ __forceinline__ void scale(float &a, float f) { a *= f; }
    static __device__ __forceinline__ void add_comp(float &s, float &c, const float &v) { fae_add_comp(s, c, v); }
    static __device__ __forceinline__ float shfl_xor(const float &a, int m) { return __shfl_xor(a, m, FAE_WAVE); }
};

typedef float fae_v4f __attribute__((ext_vector_type(4)));
// streaming store: the pooled output is written once and not read again by this kernel
__device__ __forceinline__ void fwd_store(float4 *p, const float4 &v, bool stream)
{
    if (stream)
        __builtin_nontemporal_store(*(const fae_v4f *)&v, (fae_v4f *)p);
    else
        *p = v;
}
__device__ __forceinline__ void fwd_store(float *p, const float &v, bool stream)
{
    if (stream)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// One-hot tables (one lookup per sample): a wave takes 64 consecutive samples starting at s0,
// reads their 64 slots with one coalesced load and then copies rows, 64/LPR rows per step, with
// the loads of up to 16 steps in flight before the first store.  obase points at the table's
// first output column of sample 0.
template <typename V, int LPR>
__device__ __forceinline__ void fwd_onehot_wave(const V *W, const int32_t *slots, int n_hot, int64_t s0, int n_samples,
                                                float *obase, int64_t out_stride, int dim, uint32_t *status,
                                                bool stream_out)
{
    constexpr int G = FAE_WAVE / LPR;
    constexpr int STEPS = FAE_WAVE / G;
    constexpr int UN = STEPS < 16 ? STEPS : 16;
    const int lane = fae_lane(), g = lane / LPR, l = lane % LPR;
    if (s0 >= n_samples)
        return;
    int sreg = -1;
    if (s0 + lane < n_samples) {
        sreg = slots[s0 + lane];
        if ((unsigned)sreg >= (unsigned)n_hot) {
            fae_flag(status, FAE_STATUS_ERANGE);
            sreg = -1; // pooled row of an invalid slot: zeros
        }
    }
    const int ncols = dim / (int)(sizeof(V) / sizeof(float));
    for (int c0 = 0; c0 < ncols; c0 += LPR) {
        const int c = c0 + l;
        const bool active = c < ncols;
#pragma unroll
        for (int i0 = 0; i0 < STEPS; i0 += UN) {
            V v[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int sl = __shfl(sreg, (i0 + u) * G + g, FAE_WAVE);
                v[u] = (active && sl >= 0) ? W[(int64_t)sl * ncols + c] : vec_ops<V>::zero();
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int64_t s = s0 + (i0 + u) * G + g;
                if (active && s < n_samples)
                    fwd_store((V *)(obase + s * out_stride) + c, v[u], stream_out);
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// Sort of one part of a small table inside LDS: the workgroup loads all n (<= LSORT_MAX)
// keys of the table (64 KiB of LDS, left in place), takes the keys whose top bits
// (key >> pshift) equal `part` (an ordered selection, so the input order survives) and
// LSD-sorts that subset on the remaining low bits.  What moves is a 16-bit permutation
// (position -> original lookup), ping-ponged between two 32 KiB arrays.  A radix pass makes
// two sweeps over the permutation: a per-wave digit histogram, then a stable ranking
// (wave-level match on the digit, running per-wave offsets).  Parts are disjoint key ranges,
// so their outputs are laid end to end: a part starts after all keys of lower parts.
// keys_out / vals_out point at the table's segment.  Needs LSORT_THREADS threads.
// ---------------------------------------------------------------------------------
#define LSORT_THREADS 1024
#define LSORT_WAVES (LSORT_THREADS / FAE_WAVE)
#define LSORT_MAX 16384
#define LSORT_MAX_BLOCKS 1024

// LSD radix passes inside LDS on a 16-bit permutation: perm0[0..n_sel) holds indices into
// `keys`; sorts them stably by the low `nbits` bits of (keys[idx] - sub), ping-ponging between
// perm0 and perm1.  Returns 0 / 1: which of the two holds the result.  A pass makes two sweeps:
// a per-wave digit histogram (one LDS atomic per run of equal digits), then a stable ranking
// (wave-level match on the digit, running per-wave offsets).  All LSORT_THREADS threads call it.
__device__ __forceinline__ int lds_radix_passes(const int *keys, int sub, int n_sel, int nbits, unsigned short *perm0,
                                                unsigned short *perm1, int (*wcnt)[RADIX], int *scan_lds)
{
    const int w = threadIdx.x / FAE_WAVE, lane = fae_lane();
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    const int passes = (nbits + RADIX_BITS - 1) / RADIX_BITS;
    const int digit_bits = passes > 0 ? (nbits + passes - 1) / passes : RADIX_BITS;
    const int mask = (1 << digit_bits) - 1;
    const int rounds = (n_sel + LSORT_THREADS - 1) / LSORT_THREADS; // 64-element rounds per wave
    const int wbase = w * rounds * FAE_WAVE + lane;
    volatile int *my_cnt = wcnt[w];
    int cur = 0;
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = pass * digit_bits;
        const unsigned short *src = cur ? perm1 : perm0;
        unsigned short *dst = cur ? perm0 : perm1;
#pragma unroll
        for (int i = 0; i < RADIX / FAE_WAVE; ++i)
            wcnt[w][i * FAE_WAVE + lane] = 0;
        __builtin_amdgcn_wave_barrier();
        // sweep 1: digit histogram of the positions this wave owns
        for (int i = 0; i < rounds; ++i) {
            const int pos = wbase + i * FAE_WAVE;
            const bool valid = pos < n_sel;
            const int d = valid ? ((keys[src[pos]] - sub) >> shift) & mask : -1;
            const int dprev = __shfl_up(d, 1, FAE_WAVE);
            const bool head = valid && (lane == 0 || dprev != d);
            const uint64_t heads = __ballot(head) | ((__ballot(!valid) & (0 - __ballot(!valid))));
            if (head) {
                const uint64_t later = lane == FAE_WAVE - 1 ? 0ull : (heads >> (lane + 1));
                const int len = later ? __builtin_ctzll(later) + 1 : FAE_WAVE - lane;
                atomicAdd(&wcnt[w][d], len);
            }
        }
        __syncthreads();
        // digit t: counts -> exclusive prefix over (digit, wave)
        int total = 0;
        if (threadIdx.x < RADIX) {
            for (int ww = 0; ww < LSORT_WAVES; ++ww) {
                const int c = wcnt[ww][threadIdx.x];
                wcnt[ww][threadIdx.x] = total;
                total += c;
            }
        }
        int all;
        const int ex = fae_block_excl_scan<LSORT_THREADS>(total, scan_lds, &all);
        if (threadIdx.x < RADIX) {
            for (int ww = 0; ww < LSORT_WAVES; ++ww)
                wcnt[ww][threadIdx.x] += ex;
        }
        __syncthreads();
        // sweep 2: stable ranks, running offsets per wave and digit
        for (int i = 0; i < rounds; ++i) {
            const int pos = wbase + i * FAE_WAVE;
            const bool valid = pos < n_sel;
            const int e = valid ? src[pos] : 0;
            const int d = valid ? ((keys[e] - sub) >> shift) & mask : 0;
            uint64_t peers = __ballot(valid);
#pragma unroll
            for (int b = 0; b < RADIX_BITS; ++b) {
                if (b >= digit_bits)
                    break; // the digits of this sort are narrower than a byte
                const bool bit = (d >> b) & 1;
                const uint64_t m = __ballot(bit);
                peers &= bit ? m : ~m;
            }
            const int r = __popcll(peers & lt_mask);
            const int n_peers = __popcll(peers);
            if (valid) {
                const int old = my_cnt[d];
                if (r == 0)
                    my_cnt[d] = old + n_peers;
                dst[old + r] = (unsigned short)e;
            }
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
        cur ^= 1;
    }
    return cur;
}

__device__ __forceinline__ void lds_sort_block(const int32_t *slots, const int32_t *off, int n, int n_hot, int part,
                                               int pshift, int n_samples, int32_t *keys_out, int32_t *vals_out,
                                               uint32_t *status, bool unordered)
{
    __shared__ __align__(16) int keyA[LSORT_MAX];
    __shared__ unsigned short perm[2][LSORT_MAX];
    __shared__ int wcnt[LSORT_WAVES][RADIX];
    __shared__ int scan_lds[LSORT_THREADS / FAE_WAVE + 1];
    const int w = threadIdx.x / FAE_WAVE, lane = fae_lane();

    // Every key of the table, sixteen consecutive lookups per thread: the keys go to LDS (the
    // passes below fetch them by position) and stay in registers for the ordered selection of
    // this part's lookups, which then needs no sweep over LDS: a thread's selected positions
    // follow those of all threads before it.
    constexpr int PER = LSORT_MAX / LSORT_THREADS;
    int kk[PER];
    const int e0 = threadIdx.x * PER;
    if (e0 + PER <= n && (((uintptr_t)slots) & 15) == 0) {
#pragma unroll
        for (int i = 0; i < PER; i += 4) {
            const int4 t = *(const int4 *)(slots + e0 + i);
            kk[i] = t.x; kk[i + 1] = t.y; kk[i + 2] = t.z; kk[i + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < PER; ++i)
            kk[i] = e0 + i < n ? slots[e0 + i] : 0;
    }
    bool bad = false;
    int below = 0, mine = 0; // this thread's keys in lower parts (they precede this part's output) / in this part
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        if (e0 + i < n) {
            if ((unsigned)kk[i] >= (unsigned)n_hot) {
                bad = true;
                kk[i] = n_hot; // behind every valid slot; never dereferenced
            }
            const int pk = kk[i] >> pshift;
            below += pk < part ? 1 : 0;
            mine += pk == part ? 1 : 0;
        } else {
            kk[i] = -1; // in no part
        }
    }
    if (unordered && pshift < 31 && (1 << pshift) <= LSORT_MAX) {
        // Counting sort: one counter per slot of the part's range (they take the place of the keys in
        // LDS; the keys stay in registers), a scan, and every lookup takes the next free place of its
        // slot.  One sweep each way instead of two ranked radix passes; which lookup of a slot gets
        // which place is left to the order in which the LDS serves the atomics.
        int *cnt = keyA;
        const int range = 1 << pshift, lo = part << pshift;
        for (int i = threadIdx.x; i < range; i += LSORT_THREADS)
            cnt[i] = 0;
        if (bad && part == 0)
            fae_flag(status, FAE_STATUS_ERANGE);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (kk[i] >= 0 && (kk[i] >> pshift) == part)
                atomicAdd(&cnt[kk[i] - lo], 1);
        int n_below;
        (void)fae_block_excl_scan<LSORT_THREADS>(below, scan_lds, &n_below); // its barriers also end the counting
        const int per = (range + LSORT_THREADS - 1) / LSORT_THREADS; // counters per thread, <= PER
        int c[PER], own = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int r = threadIdx.x * per + i;
            c[i] = (i < per && r < range) ? cnt[r] : 0;
            own += c[i];
        }
        int n_part;
        int at = fae_block_excl_scan<LSORT_THREADS>(own, scan_lds, &n_part);
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int r = threadIdx.x * per + i;
            if (i < per && r < range)
                cnt[r] = at;
            at += c[i];
        }
        __syncthreads();
        bad = false;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (kk[i] < 0 || (kk[i] >> pshift) != part)
                continue;
            const int e = e0 + i;
            int sm = e;
            if (off) {
                sm = fae_sample_of(off, n_samples, e);
                if (off[sm] > e || off[sm + 1] <= e)
                    bad = true; // malformed CSR
            }
            const int place = n_below + atomicAdd(&cnt[kk[i] - lo], 1);
            keys_out[place] = kk[i];
            vals_out[place] = sm;
        }
        if (bad)
            fae_flag(status, FAE_STATUS_ERANGE);
        return;
    }
#pragma unroll
    for (int i = 0; i < PER; i += 4)
        if (e0 + i < n) // keyA is a multiple of four keys long, so a ragged end may write past n
            *(int4 *)(keyA + e0 + i) = make_int4(kk[i], kk[i + 1], kk[i + 2], kk[i + 3]);
    if (bad && part == 0)
        fae_flag(status, FAE_STATUS_ERANGE);
    // one scan for both counts (each at most LSORT_MAX = 2^14)
    int n_below, n_sel;
    {
        int both;
        const int ex = fae_block_excl_scan<LSORT_THREADS>((below << 16) | mine, scan_lds, &both);
        n_below = both >> 16;
        n_sel = both & 0xffff;
        int at = ex & 0xffff;
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (kk[i] >= 0 && (kk[i] >> pshift) == part)
                perm[0][at++] = (unsigned short)(e0 + i);
    }
    __syncthreads();

    // LSD passes over the bits below part_shift
    const int cur = lds_radix_passes(keyA, 0, n_sel, pshift, perm[0], perm[1], wcnt, scan_lds);
    const int out0 = n_below;
    const unsigned short *fin = perm[cur];
    bad = false;
    for (int pos = threadIdx.x; pos < n_sel; pos += LSORT_THREADS) {
        const int e = fin[pos];
        int s = e;
        if (off) {
            s = fae_sample_of(off, n_samples, e);
            if (off[s] > e || off[s + 1] <= e)
                bad = true; // malformed CSR
        }
        keys_out[out0 + pos] = keyA[e];
        vals_out[out0 + pos] = s;
    }
    if (bad)
        fae_flag(status, FAE_STATUS_ERANGE);
}

