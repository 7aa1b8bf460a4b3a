// Device-side helpers: wave-wide reductions and the Online Correction Memory slot operations.
#pragma once

#include "csd_internal.h"

namespace csd {

// ---- wave-wide all-reduces: DPP inside a row of 16 lanes, ds_swizzle across rows, bpermute across halves.
// Every lane ends up with the result (both partners of a step compute op(own, other), and op is commutative).
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ int xor16_i(int v) { return __builtin_amdgcn_ds_swizzle(v, 0x401F); }   // lane ^ 16
__device__ __forceinline__ int xor32_i(int v) {
    return __builtin_amdgcn_ds_bpermute(((int)__lane_id() ^ 32) << 2, v);
}

template <typename Op>
__device__ __forceinline__ float wave_allreduce_f(float v, Op op) {
    v = op(v, __int_as_float(dpp_i<0xB1>(__float_as_int(v))));    // quad_perm [1,0,3,2]
    v = op(v, __int_as_float(dpp_i<0x4E>(__float_as_int(v))));    // quad_perm [2,3,0,1]
    v = op(v, __int_as_float(dpp_i<0x141>(__float_as_int(v))));   // row_half_mirror (quads are uniform now)
    v = op(v, __int_as_float(dpp_i<0x140>(__float_as_int(v))));   // row_mirror      (halves are uniform now)
    v = op(v, __int_as_float(xor16_i(__float_as_int(v))));
    v = op(v, __int_as_float(xor32_i(__float_as_int(v))));
    return v;
}
template <typename Op>
__device__ __forceinline__ int wave_allreduce_i(int v, Op op) {
    v = op(v, dpp_i<0xB1>(v));
    v = op(v, dpp_i<0x4E>(v));
    v = op(v, dpp_i<0x141>(v));
    v = op(v, dpp_i<0x140>(v));
    v = op(v, xor16_i(v));
    v = op(v, xor32_i(v));
    return v;
}
struct MaxF { __device__ float operator()(float a, float b) const { return __builtin_fmaxf(a, b); } };
struct AddF { __device__ float operator()(float a, float b) const { return a + b; } };
struct MinI { __device__ int operator()(int a, int b) const { return a < b ? a : b; } };

// lane ^ mask exchange for any mask < 64 (bpermute); used off the hot loop only
__device__ __forceinline__ int xchg_i(int v, int mask) {
    return __builtin_amdgcn_ds_bpermute(((int)__lane_id() ^ mask) << 2, v);
}
__device__ __forceinline__ float xchg_f(float v, int mask) { return __int_as_float(xchg_i(__float_as_int(v), mask)); }
__device__ __forceinline__ double xchg_d(double v, int mask) {
    const long long b = __double_as_longlong(v);
    const int lo = xchg_i((int)(b & 0xFFFFFFFFll), mask), hi = xchg_i((int)(b >> 32), mask);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
// value held by lane `src`
__device__ __forceinline__ int from_lane_i(int v, int src) { return __builtin_amdgcn_ds_bpermute(src << 2, v); }
__device__ __forceinline__ float from_lane_f(float v, int src) { return __int_as_float(from_lane_i(__float_as_int(v), src)); }
__device__ __forceinline__ double from_lane_d(double v, int src) {
    const long long b = __double_as_longlong(v);
    const int lo = from_lane_i((int)(b & 0xFFFFFFFFll), src), hi = from_lane_i((int)(b >> 32), src);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// ---- Online Correction Memory slots (layout in csd.h)
__device__ __forceinline__ uint64_t slot_key(uint64_t s) { return s & CSD_OCM_KEY_MASK; }
__device__ __forceinline__ uint32_t slot_count(uint64_t s) { return (uint32_t)(s >> CSD_OCM_KEY_BITS); }

// Fibonacci hashing of the 40-bit key; capacity is a power of two.
__device__ __forceinline__ uint64_t home_slot(uint64_t key, uint64_t capacity) {
    const uint64_t h = key * 0x9E3779B97F4A7C15ull;
    return (h >> 20) & (capacity - 1);
}

// T[key], 0 if absent.  Linear probing; an empty slot ends the search (there is no deletion).
__device__ inline uint32_t ocm_lookup(const uint64_t *ocm, uint64_t capacity, uint64_t key) {
    uint64_t i = home_slot(key, capacity);
    for (uint64_t probe = 0; probe < capacity; ++probe) {
        const uint64_t s = __hip_atomic_load(&ocm[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint64_t sk = slot_key(s);
        if (sk == key) return slot_count(s);
        if (sk == CSD_OCM_EMPTY) return 0;
        i = (i + 1) & (capacity - 1);
    }
    return 0;
}

// T[key] += w (saturating), inserting the key if absent.  Returns false when every slot holds another key.
__device__ inline bool ocm_add(uint64_t *ocm, uint64_t capacity, uint64_t key, uint32_t w) {
    uint64_t i = home_slot(key, capacity);
    for (uint64_t probe = 0; probe < capacity; ++probe) {
        uint64_t cur = __hip_atomic_load(&ocm[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (;;) {
            const uint64_t ck = slot_key(cur);
            if (ck != key && ck != CSD_OCM_EMPTY) break;              // another pair lives here: next slot
            uint64_t cnt = (ck == key) ? (uint64_t)slot_count(cur) : 0ull;
            cnt += w;
            if (cnt > CSD_OCM_COUNT_MAX) cnt = CSD_OCM_COUNT_MAX;
            const uint64_t want = key | (cnt << CSD_OCM_KEY_BITS);
            if (__hip_atomic_compare_exchange_strong(&ocm[i], &cur, want, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT))
                return true;
            // lost a race: `cur` now holds the slot's new content; look at it again
        }
        i = (i + 1) & (capacity - 1);
    }
    return false;
}

// Where a lookup ended: at the pair's slot (found, with its count), at the empty slot that ends its probe
// chain (the slot an insert would try first), or nowhere (every slot holds another pair).  Slots are never
// freed or moved, so a found slot stays the pair's slot for the life of the table.
struct OcmProbe {
    uint64_t slot;
    uint32_t count;
    bool found;
    bool full;
};
__device__ inline OcmProbe ocm_probe(const uint64_t *ocm, uint64_t capacity, uint64_t key) {
    OcmProbe r;
    r.slot = home_slot(key, capacity);
    r.count = 0;
    r.found = false;
    r.full = false;
    for (uint64_t probe = 0; probe < capacity; ++probe) {
        const uint64_t s = __hip_atomic_load(&ocm[r.slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint64_t sk = slot_key(s);
        if (sk == key) {
            r.found = true;
            r.count = slot_count(s);
            return r;
        }
        if (sk == CSD_OCM_EMPTY) return r;
        r.slot = (r.slot + 1) & (capacity - 1);
    }
    r.full = true;
    return r;
}

// First half of an insert, usable before the step's other lookups have finished: claim the empty slot the probe
// ended at for `key`, with count ZERO.  A pair that is absent and a pair that is present with count zero read
// the same in every lookup, so this changes no decision of the step; the count is added later.  The result
// (`won`, and what the slot held otherwise) is first looked at in ocm_add_after_claim, so the
// compare-and-swap can stay in flight while the caller does other things.
struct OcmClaim {
    uint64_t seen;       // content of the slot when the claim lost
    bool tried, won;
};
__device__ __forceinline__ OcmClaim ocm_claim_after_probe(uint64_t *ocm, uint64_t key, const OcmProbe &pr) {
    OcmClaim c;
    c.seen = CSD_OCM_EMPTY;
    c.tried = !pr.found && !pr.full;
    c.won = false;
    if (c.tried)
        c.won = __hip_atomic_compare_exchange_strong(&ocm[pr.slot], &c.seen, key, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
    return c;
}

constexpr uint32_t kHintHeadroom = 1u << 20;   // increments by others allowed for between a probe and the add that uses it

// Second half: the pair sits at pr.slot (found by the probe, or claimed there since - by this lane or, a moment
// ago, by another lane of the step) and takes one atomic add of w (a workgroup's occurrences of the pair, far below
// the headroom); anything else goes the general way.
__device__ inline bool ocm_add_after_claim(uint64_t *ocm, uint64_t capacity, uint64_t key, uint32_t w, const OcmProbe &pr,
                                           const OcmClaim &c) {
    const bool here = (pr.found && pr.count < CSD_OCM_COUNT_MAX - kHintHeadroom) ||
                      (c.tried && (c.won || (slot_key(c.seen) == key && slot_count(c.seen) < CSD_OCM_COUNT_MAX - kHintHeadroom)));
    if (here) {
        __hip_atomic_fetch_add(&ocm[pr.slot], (uint64_t)w << CSD_OCM_KEY_BITS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    return ocm_add(ocm, capacity, key, w);
}

// A workgroup barrier that waits for LDS traffic only: values handed round through LDS are complete, stores and
// atomics to global memory may still be in flight (a plain __syncthreads waits for every one of them to be
// acknowledged, a memory round trip).  The empty asm statements keep the compiler from moving memory
// operations across it.
__device__ __forceinline__ void barrier_lds_only() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);             // lgkmcnt(0); vmcnt and expcnt left alone
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// ---- applying a list of (key, weight) entries to the table, one workgroup of kApplyThreads threads.
// Entries are merged in an LDS hash table first, kApplyBatch at a time, so a skewed list costs one
// compare-and-swap chain per DISTINCT pair; the distinct pairs are then compacted so that all of them
// go to the table side by side (one round of global atomics per kApplyThreads distinct pairs) instead of
// slot by slot.
constexpr int kApplyThreads = 1024;               // also the finish kernels' workgroup: 16 sequences each
constexpr int kApplyBatch = 1024;                 // entries merged at a time
constexpr int kApplySlots = 2 * kApplyBatch;      // LDS table never fills
constexpr int kApplyPerThread = kApplyBatch / kApplyThreads;

struct ApplyLds {
    unsigned long long key[kApplySlots];
    unsigned long long cnt[kApplySlots];          // 64-bit: sums of weights of up to 2^24-1 do not wrap
    unsigned long long ckey[kApplySlots];         // compacted distinct pairs ...
    unsigned long long ccnt[kApplySlots];         // ... and their summed weights
    unsigned int nkeys;                           // distinct pairs in the table
    unsigned int ndistinct;                       // length of the compacted list
};

__device__ __forceinline__ void lds_aggregate(ApplyLds &L, uint64_t key, uint32_t w) {
    uint32_t i = (uint32_t)((key * 0x9E3779B97F4A7C15ull) >> 40) & (kApplySlots - 1);
    for (;;) {
        unsigned long long cur = L.key[i];
        if (cur == CSD_OCM_EMPTY) {
            cur = atomicCAS(&L.key[i], (unsigned long long)CSD_OCM_EMPTY, (unsigned long long)key);
            if (cur == CSD_OCM_EMPTY) atomicAdd(&L.nkeys, 1u);      // this thread put the pair in
        }
        if (cur == CSD_OCM_EMPTY || cur == key) {
            atomicAdd(&L.cnt[i], (unsigned long long)w);
            return;
        }
        i = (i + 1) & (kApplySlots - 1);
    }
}

// The three steps below are called by every thread of the workgroup (they contain barriers).
__device__ __forceinline__ void block_apply_clear(ApplyLds &L) {
    for (int i = threadIdx.x; i < kApplySlots; i += kApplyThreads) {
        L.key[i] = CSD_OCM_EMPTY;
        L.cnt[i] = 0;
    }
    if (threadIdx.x == 0) {
        L.nkeys = 0;
        L.ndistinct = 0;
    }
    __syncthreads();
}
// the table's pairs go to the memory, all of them side by side; the table is left empty when it is to be used again
__device__ __forceinline__ void block_apply_flush(uint64_t *ocm, uint64_t capacity, uint32_t *status, ApplyLds &L,
                                                  bool use_again) {
    const int tid = threadIdx.x;
    __syncthreads();
    for (int i = tid; i < kApplySlots; i += kApplyThreads) {
        const unsigned long long sk = L.key[i];
        if (sk != CSD_OCM_EMPTY) {
            const unsigned int pos = atomicAdd(&L.ndistinct, 1u);
            L.ckey[pos] = sk;
            L.ccnt[pos] = L.cnt[i];
        }
    }
    __syncthreads();
    const unsigned int nd = L.ndistinct;
    for (unsigned int i = tid; i < nd; i += kApplyThreads) {
        const unsigned long long sum = L.ccnt[i];
        const uint32_t ww = (sum > CSD_OCM_COUNT_MAX) ? CSD_OCM_COUNT_MAX : (uint32_t)sum;
        if (!ocm_add(ocm, capacity, L.ckey[i], ww) && status) atomicAdd(&status[CSD_STATUS_DROPPED], ww);
    }
    if (use_again) {
        __syncthreads();
        block_apply_clear(L);
    }
}

// Batches first, first + stride, ... (of kApplyBatch entries each) of a list of n entries; fetch(e, key, w) reads
// entry e.  Entries with an empty key or zero weight are skipped.  The LDS table keeps merging across batches
// and is emptied into the memory only when the next batch might not fit, and at the end: a workgroup that
// meets the same few pairs over and over sends each of them once.
template <typename Fetch>
__device__ __forceinline__ void block_apply_list(uint64_t *ocm, uint64_t capacity, uint32_t *status, ApplyLds &L, Fetch fetch,
                                                 uint64_t first, uint64_t stride, uint64_t n) {
    const int tid = threadIdx.x;
    block_apply_clear(L);
    for (uint64_t base = first * kApplyBatch; base < n; base += stride * kApplyBatch) {
        uint64_t key[kApplyPerThread];
        uint32_t w[kApplyPerThread];
#pragma unroll
        for (int j = 0; j < kApplyPerThread; ++j) {     // all global reads first: their latencies overlap
            const uint64_t e = base + (uint64_t)(j * kApplyThreads + tid);
            key[j] = CSD_OCM_EMPTY;
            w[j] = 0;
            if (e < n) fetch(e, key[j], w[j]);
        }
        // Every thread must take the same branch (the flush has barriers): all read the count before anyone
        // adds to it again.
        const unsigned int have = L.nkeys;
        __syncthreads();
        if (have + kApplyBatch > (unsigned int)(kApplySlots - kApplySlots / 4)) block_apply_flush(ocm, capacity, status, L, true);
#pragma unroll
        for (int j = 0; j < kApplyPerThread; ++j)
            if (key[j] != CSD_OCM_EMPTY && w[j] != 0) lds_aggregate(L, key[j], w[j]);
        __syncthreads();                                // nkeys is read by every thread at the top of the next round
    }
    block_apply_flush(ocm, capacity, status, L, false);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---- 16-byte chunk of logits -> fp32 values (bf16 widening is exact)
template <int DT> struct Chunk;
template <> struct Chunk<CSD_DTYPE_F32> {
    static constexpr int E = 4;
    static constexpr uint32_t kNegInfWord = 0xFF800000u;
    __device__ static __forceinline__ void unpack(const u32x4 &q, float (&x)[E]) {
        x[0] = __uint_as_float(q.x); x[1] = __uint_as_float(q.y);
        x[2] = __uint_as_float(q.z); x[3] = __uint_as_float(q.w);
    }
    // the last, partial chunk of a row: n < E logits starting at element v0, the rest -inf
    __device__ static __forceinline__ u32x4 load_ragged(const char *row, int v0, int n) {
        const uint32_t *p = (const uint32_t *)row + v0;
        u32x4 q = {kNegInfWord, kNegInfWord, kNegInfWord, kNegInfWord};
        if (n > 0) q.x = p[0];
        if (n > 1) q.y = p[1];
        if (n > 2) q.z = p[2];
        return q;
    }
};
template <> struct Chunk<CSD_DTYPE_BF16> {
    static constexpr int E = 8;
    static constexpr uint32_t kNegInfWord = 0xFF80FF80u;
    __device__ static __forceinline__ void unpack(const u32x4 &q, float (&x)[E]) {
        x[0] = __uint_as_float(q.x << 16); x[1] = __uint_as_float(q.x & 0xFFFF0000u);
        x[2] = __uint_as_float(q.y << 16); x[3] = __uint_as_float(q.y & 0xFFFF0000u);
        x[4] = __uint_as_float(q.z << 16); x[5] = __uint_as_float(q.z & 0xFFFF0000u);
        x[6] = __uint_as_float(q.w << 16); x[7] = __uint_as_float(q.w & 0xFFFF0000u);
    }
    __device__ static __forceinline__ u32x4 load_ragged(const char *row, int v0, int n) {
        const uint16_t *p = (const uint16_t *)row + v0;
        uint32_t w[4] = {kNegInfWord, kNegInfWord, kNegInfWord, kNegInfWord};
#pragma unroll
        for (int j = 0; j < 7; ++j) {
            if (j < n) {
                const uint32_t h = p[j];
                w[j >> 1] = (j & 1) ? ((w[j >> 1] & 0x0000FFFFu) | (h << 16)) : ((w[j >> 1] & 0xFFFF0000u) | h);
            }
        }
        u32x4 q = {w[0], w[1], w[2], w[3]};
        return q;
    }
};

template <int E>
__device__ __forceinline__ float chunk_max(const float (&x)[E]) {
    float m = x[0];
#pragma unroll
    for (int j = 1; j < E; ++j) m = __builtin_fmaxf(m, x[j]);
    return m;
}

// ---- data handed between workgroups: agent-scope relaxed atomics, 64 bits at a time
__device__ __forceinline__ void xwg_store64(uint64_t *p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t xwg_load64(const uint64_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// One atomic ticket per workgroup: true in every thread of the workgroup that drew the last of `total`
// tickets.  Every wave first waits until its own vector-memory operations are acknowledged
// (s_waitcnt vmcnt(0): on gfx9 the counter covers stores, and a write-through store is acknowledged once
// it is visible at agent scope) - a workgroup barrier alone does not wait for them.  The second barrier
// hands the verdict round; the reads of the log depend on it, so they cannot be issued early.
// The workgroup-scope fences cost no cache maintenance; they keep the compiler from moving the log's stores
// below the ticket or the log's loads above the verdict.
__device__ __forceinline__ bool take_last_ticket(uint32_t *ticket, uint32_t total, int *verdict) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0); expcnt and lgkmcnt left alone
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t old = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *verdict = (old == total - 1);
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return *verdict != 0;
}

// ---------------------------------------------------------------------------------------------------
// Combine the partials of one row, shared by a group of G lanes (G a power of two; lane gs of the group
// takes partials gs, gs+G, ...).  Two passes over the partials (the second finds them in cache): first the
// maximum m and its lowest token id t, a butterfly over the group; then S = sum s_j 2^(cref_j - m*scale)
// against that one maximum - independent terms in double - and a second butterfly.  `scale` is the exponent
// scale the partials were made with (log2e / temperature), as a double holding the float value.  A row
// may come as several sets of partials (vocabulary shards, token ids offset by the shard's base): the
// `*_pass` functions take one set each, the `*_merge` functions finish a pass across the group.
// Both passes read four partials per lane at a time, all four loads issued before any is used: a plain
// loop would pay one memory latency per partial.
constexpr int kPartialBatch = 4;
__device__ __forceinline__ RowPartial empty_partial() {
    RowPartial q;
    q.m = -INFINITY;
    q.cref = 0.f;
    q.s = 0.f;
    q.idx = 0x7fffffff;
    return q;
}
__device__ __forceinline__ void partials_max_pass(const RowPartial *pp, int P, int G, int gs, int idx_base, float &gm, int &t) {
    for (int j0 = gs; j0 < P; j0 += kPartialBatch * G) {
        RowPartial q[kPartialBatch];
#pragma unroll
        for (int u = 0; u < kPartialBatch; ++u) q[u] = (j0 + u * G < P) ? pp[j0 + u * G] : empty_partial();
#pragma unroll
        for (int u = 0; u < kPartialBatch; ++u) {
            const int qi = (q[u].idx == 0x7fffffff) ? q[u].idx : q[u].idx + idx_base;
            if (q[u].m > gm || (q[u].m == gm && qi < t)) t = qi;
            gm = fmaxf(gm, q[u].m);
        }
    }
}
__device__ __forceinline__ void partials_max_merge(int G, float &gm, int &t) {
    for (int x = 1; x < G; x <<= 1) {
        const float om = xchg_f(gm, x);
        const int ot = xchg_i(t, x);
        if (om > gm || (om == gm && ot < t)) t = ot;
        gm = fmaxf(gm, om);
    }
}
__device__ __forceinline__ void partials_sum_pass(const RowPartial *pp, int P, int G, int gs, double mref, double &S) {
    for (int j0 = gs; j0 < P; j0 += kPartialBatch * G) {
        RowPartial q[kPartialBatch];
#pragma unroll
        for (int u = 0; u < kPartialBatch; ++u) q[u] = (j0 + u * G < P) ? pp[j0 + u * G] : empty_partial();
#pragma unroll
        for (int u = 0; u < kPartialBatch; ++u) {
            // the exponent difference is exact in double; as a float it is off by at most 2^-24 of itself, which
            // only matters for terms too small to count, so the hardware exp2 serves
            if (q[u].s != 0.f) S += (double)q[u].s * (double)__builtin_amdgcn_exp2f((float)((double)q[u].cref - mref));
        }
    }
}
__device__ __forceinline__ void partials_sum_merge(int G, double &S) {
    for (int x = 1; x < G; x <<= 1) S += xchg_d(S, x);
}
// A row whose partials fit NB registers per lane (the usual case) is read ONCE, all loads in flight together.
// the arithmetic of the combine on partials already in registers (unused entries = empty_partial())
template <int NB>
__device__ __forceinline__ void combine_partials_in_registers(const RowPartial (&q)[NB], int G, double scale, float &gm, int &t,
                                                              double &S);
template <int NB>
__device__ __forceinline__ void combine_row_partials_once(const RowPartial *pp, int P, int G, int gs, double scale, float &gm,
                                                          int &t, double &S) {
    RowPartial q[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) q[u] = (gs + u * G < P) ? pp[gs + u * G] : empty_partial();
    combine_partials_in_registers<NB>(q, G, scale, gm, t, S);
}
template <int NB>
__device__ __forceinline__ void combine_partials_in_registers(const RowPartial (&q)[NB], int G, double scale, float &gm, int &t,
                                                              double &S) {
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        if (q[u].m > gm || (q[u].m == gm && q[u].idx < t)) t = q[u].idx;
        gm = fmaxf(gm, q[u].m);
    }
    partials_max_merge(G, gm, t);
    const double mref = (double)gm * scale;                    // exact: two 24-bit significands
#pragma unroll
    for (int u = 0; u < NB; ++u)
        if (q[u].s != 0.f) S += (double)q[u].s * (double)__builtin_amdgcn_exp2f((float)((double)q[u].cref - mref));
    partials_sum_merge(G, S);
}
__device__ __forceinline__ void combine_row_partials(const RowPartial *pp, int P, int G, int gs, double scale, float &gm,
                                                     int &t, double &S) {
    gm = -INFINITY;
    t = 0x7fffffff;
    S = 0.0;
    const int per_lane = (P + G - 1) / G;                      // wave-uniform
    if (per_lane <= 2) return combine_row_partials_once<2>(pp, P, G, gs, scale, gm, t, S);
    if (per_lane <= 4) return combine_row_partials_once<4>(pp, P, G, gs, scale, gm, t, S);
    if (per_lane <= 9) return combine_row_partials_once<9>(pp, P, G, gs, scale, gm, t, S);
    if (per_lane <= 16) return combine_row_partials_once<16>(pp, P, G, gs, scale, gm, t, S);
    partials_max_pass(pp, P, G, gs, 0, gm, t);
    partials_max_merge(G, gm, t);
    partials_sum_pass(pp, P, G, gs, (double)gm * scale, S);     // m * scale is exact: two 24-bit significands
    partials_sum_merge(G, S);
}

// Status counters of a step are summed per workgroup in LDS and leave it as one global atomic per counter:
// hundreds of waves adding to the same four words cost the finish kernels several microseconds.
struct BlockCounters {
    unsigned int v[CSD_STATUS_WORDS];
};
__device__ __forceinline__ void block_counters_clear(BlockCounters &c) {     // every thread; contains a barrier
    if (threadIdx.x < CSD_STATUS_WORDS) c.v[threadIdx.x] = 0;
    __syncthreads();
}
__device__ __forceinline__ void block_counters_flush(BlockCounters &c, uint32_t *status) {   // every thread; barrier
    __syncthreads();
    if (status != nullptr && threadIdx.x < CSD_STATUS_WORDS && c.v[threadIdx.x] != 0)
        atomicAdd(&status[threadIdx.x], c.v[threadIdx.x]);
}

// The tail of a step: the workgroup that draws the last of gridDim.x tickets applies the step's log of n
// entries (every lookup of the step has then been made).  Called by every thread of every workgroup.
constexpr int kFinishWaves = kApplyThreads / kWaveSize;
__device__ __forceinline__ void apply_step_log(uint64_t *ocm, uint64_t capacity, uint32_t *status, const uint64_t *rej_log,
                                               uint64_t n, uint32_t *ticket, ApplyLds &lds, int *verdict) {
    if (!take_last_ticket(ticket, gridDim.x, verdict)) return;
    auto fetch = [&](uint64_t e, uint64_t &key, uint32_t &w) {
        key = xwg_load64(&rej_log[e]) & CSD_OCM_KEY_MASK;
        w = 1u;
    };
    block_apply_list(ocm, capacity, status, lds, fetch, 0, 1, n);
}


// ---------------------------------------------------------------------------------------------------
// Waiting inside a launch: waves that wait for what other workgroups of the same launch publish.  Every wait is
// bounded: kSpinLimit polls of about a microsecond each (a poll is a memory round trip plus a short sleep).
constexpr uint32_t kSpinLimit = 1u << 21;
constexpr int kSpinSleep = 6;                     // s_sleep units of 64 clocks between polls

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

// Divergences of one sequence workgroup that name the same pair reach the table as ONE add of their number.
// Atomic adds that meet on one address are applied one after the other where the eight XCDs agree, about 12 ns
// each (1024 adds to one word from 64 workgroups: 12.5 microseconds until the last is acknowledged; to distinct
// words: 0.7), so a step whose sequences all diverge on one pair would spend longer on its updates than on its
// logits.  A small LDS hash table, cleared when the workgroup starts, slots laid out as in the memory itself
// (count above the pair): the lane that puts a pair in is the pair's leader and adds the slot's count to the memory
// once the workgroup's barrier has passed.  Sized to hold every position of a sequence workgroup (4 waves of at
// most 63 positions); kept at 2 KiB because a workgroup of the streaming kernel that statically holds 6 KiB of LDS
// measured 0.8 microseconds slower per step on the fp32 shape (3 KiB: no difference).
constexpr int kMergeSlots = 256;
struct StepMergeLds {
    unsigned long long slot[kMergeSlots];
};
__device__ __forceinline__ void step_merge_clear(StepMergeLds &M) {   // every thread; a workgroup barrier must follow
    for (int i = threadIdx.x; i < kMergeSlots; i += blockDim.x) M.slot[i] = CSD_OCM_EMPTY;
}
// returns the pair's slot; `leader` is true in the one lane of the workgroup that put the pair there
__device__ __forceinline__ int step_merge_insert(StepMergeLds &M, uint64_t key, bool &leader) {
    uint32_t i = (uint32_t)((key * 0x9E3779B97F4A7C15ull) >> 40) & (kMergeSlots - 1);
    for (;;) {
        const unsigned long long cur = atomicCAS(&M.slot[i], (unsigned long long)CSD_OCM_EMPTY, (unsigned long long)key);
        leader = (cur == CSD_OCM_EMPTY);
        if (leader || slot_key(cur) == key) {
            atomicAdd(&M.slot[i], 1ull << CSD_OCM_KEY_BITS);
            return (int)i;
        }
        i = (i + 1) & (kMergeSlots - 1);
    }
}

// What a lane carries out of the verification loop for the update phase.
struct Divergence {
    bool counted;        // this position's pair goes to UpdateMemory
    uint64_t key;
    OcmProbe probe;      // where the lookup ended (only when probed)
    int n;               // the sequence's accepted length (wave-uniform)
};


// A sequence whose wait inside the launch ran out: nothing accepted, no emitted token, no position flagged, and
// no divergence in the log (a later bulk update must not apply what an earlier step left there).  Called by
// the sequence's wave; the caller counts it in CSD_STATUS_STALLED.
__device__ __forceinline__ void report_stalled_sequence(int32_t *accept_len, int32_t *next_token, uint8_t *pos_flags,
                                                        uint64_t *rej_log, int b, int k, int lane) {
    if (lane == 0) {
        accept_len[b] = 0;
        next_token[b] = -1;
    }
    if (lane < k) {
        const int64_t o = (int64_t)b * k + lane;
        if (pos_flags) pos_flags[o] = 0;
        if (rej_log) xwg_store64(&rej_log[o], CSD_OCM_EMPTY);
    }
}

// The end of a sequence workgroup's step, called by all its threads: the per-workgroup status counters leave
// (all but the rare lost insert are known; their atomics need no answer and travel while the workgroup waits),
// and - update_here - the step's increments are applied after a barrier of the launch's `total` sequence
// workgroups: every lookup of the step before any update of the step.
//   This workgroup's lookups have returned when it counts itself in (their values were used by the caller); its
//   stores may still be on their way, nobody waits for them.  An absent pair's slot is claimed while the barrier
//   is pending (count zero: no lookup of the step reads it differently), so the compare-and-swap and the barrier
//   share their wait.
//   The counter behind the barrier is zeroed by the first workgroup of the same launch, which then writes
//   `ready_value` (derived from the call's number) into the control head; thread 0 here asked for that word early
//   (`ready_seen`) and counts itself in only once it holds.  After the barrier every workgroup has seen it, and the
//   first sequence workgroup clears it, so that a replay of the same launch (same number) waits for its own
//   set-up; a workgroup whose wait ran out clears it as well.  Nothing here needs an answer after the barrier:
//   the increments and the clearing store travel while the kernel ends.  A launch with a single sequence
//   workgroup (up to four sequences) skips all of it: the workgroup barrier at the top already orders its
//   lookups before its updates (1.5 microseconds of a 9 microsecond step).
__device__ __forceinline__ uint64_t step_ready_value(uint64_t nonce) { return mix64(nonce ^ 0x5244595f43534431ull) | 1ull; }

__device__ __forceinline__ void sequence_counters_and_updates(StepControl *ctrl, uint64_t ready_seen, uint64_t ready_value,
                                                              bool first_sequence_workgroup, uint32_t total, bool update_here,
                                                              uint64_t *ocm, uint64_t capacity, uint32_t *status,
                                                              BlockCounters &counters, StepMergeLds &merge,
                                                              const Divergence &dv, int *verdict, uint32_t spin_limit) {
    barrier_lds_only();
    if (status != nullptr && threadIdx.x < CSD_STATUS_WORDS && counters.v[threadIdx.x] != 0)
        atomicAdd(&status[threadIdx.x], counters.v[threadIdx.x]);
    if (!update_here) return;
    bool good = true;
    const bool alone = total <= 1;                   // one sequence workgroup: its own barrier above was the barrier
    if (threadIdx.x == 0 && !alone) {
        for (uint32_t spin = 0; ready_seen != ready_value; ++spin) {
            if (spin >= spin_limit) { good = false; break; }
            __builtin_amdgcn_s_sleep(kSpinSleep);
            ready_seen = xwg_load64(&ctrl->ready);
        }
        if (good) __hip_atomic_fetch_add(&ctrl->arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    OcmClaim claim = {CSD_OCM_EMPTY, false, false};
    if (dv.counted) claim = ocm_claim_after_probe(ocm, dv.key, dv.probe);
    // while the barrier is pending: equal pairs of this workgroup find each other (step_merge_insert)
    bool leader = false;                             // this lane sends its pair's increments for the whole workgroup
    int mslot = 0;
    if (dv.counted) mslot = step_merge_insert(merge, dv.key, leader);
    if (threadIdx.x == 0) {
        if (good && !alone) {
            for (uint32_t spin = 0;; ++spin) {
                if (__hip_atomic_load(&ctrl->arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= total) break;
                if (spin >= spin_limit) { good = false; break; }
                __builtin_amdgcn_s_sleep(kSpinSleep);
            }
        }
        if (!good) {
            xwg_store64(&ctrl->ready, 0ull);
            if (status != nullptr) atomicAdd(&status[CSD_STATUS_STALLED], 1u);
        } else if (first_sequence_workgroup && !alone) {
            xwg_store64(&ctrl->ready, 0ull);
        }
        *verdict = good ? 1 : 0;
    }
    barrier_lds_only();
    if (*verdict != 0 && leader) {
        const uint32_t weight = slot_count(merge.slot[mslot]);
        if (!ocm_add_after_claim(ocm, capacity, dv.key, weight, dv.probe, claim) && status != nullptr)
            atomicAdd(&status[CSD_STATUS_DROPPED], weight);
    }
}

// The first workgroup of a launch whose sequence workgroups will use the barrier (called by one thread): the
// counter is zero, and only then does the control head say so.  The launch before has ended, nothing else
// touches the head.
__device__ __forceinline__ void step_control_setup(StepControl *ctrl, uint64_t ready_value) {
    __hip_atomic_store(&ctrl->arrivals, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): the zero is acknowledged before the word leaves
    xwg_store64(&ctrl->ready, ready_value);
}

// Published words (WordRecord): same rules as StepRecord - a reader takes one once the check holds and zeroes the
// check after use; arbitrary memory passes with probability 2^-64.
__device__ __forceinline__ uint64_t word_check(uint64_t value, uint64_t nonce, uint64_t rec) {
    return mix64(value + mix64(nonce + rec * 0x9E3779B97F4A7C15ull)) | 1ull;
}
__device__ __forceinline__ void publish_word(WordRecord *r, uint64_t nonce, uint64_t rec, uint64_t value) {
    xwg_store64(&r->value, value);
    xwg_store64(&r->check, word_check(value, nonce, rec));
}
// polled by the calling lane until it passes (bounded); false when the wait ran out
__device__ __forceinline__ bool acquire_word(WordRecord *r, uint64_t nonce, uint64_t rec, uint64_t &value, uint32_t spin_limit) {
    for (uint32_t spin = 0;; ++spin) {
        value = xwg_load64(&r->value);
        const uint64_t ck = xwg_load64(&r->check);
        if (ck == word_check(value, nonce, rec)) {
            xwg_store64(&r->check, 0ull);
            return true;
        }
        if (spin >= spin_limit) return false;
        __builtin_amdgcn_s_sleep(kSpinSleep);
    }
}

__device__ __forceinline__ float load_logit(const void *logits, int dtype, int64_t elem) {
    if (dtype == CSD_DTYPE_F32) return ((const float *)logits)[elem];
    return __uint_as_float((uint32_t)((const uint16_t *)logits)[elem] << 16);
}

}  // namespace csd
