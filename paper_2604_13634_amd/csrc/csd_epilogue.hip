// Per-sequence epilogue of the verification step and the Online Correction Memory kernels.
//
// epilogue_kernel: one wave per sequence, lane i = verify row i (draft position i, or the bonus row
// for i == k).  It
//   1. combines the row-stream partials of its row (max, lowest-id argmax, normaliser S) - the
//      normaliser in double, from partials carried with their exact reference exponents;
//   2. gathers the draft token's logit and forms ratio = exp(z_draft - m) = p(draft)/p(t*) (Eq. 3)
//      and p(draft) = ratio / S, in double;
//   3. evaluates, for a divergence, is_freq = T[(draft,t*)] >= lambda and is_safe = ratio >= tau
//      (Algorithm 1: memory lookup, then gate), by probing the table as it stands - no kernel of
//      this call has written to it yet;
//   4. finds the accepted prefix with one ballot (first position that is neither a match nor
//      rescued), the emitted extra token, and the divergences to count: every processed one,
//      rescued or not (Algorithm 1, UpdateMemory).
// The counted pairs go to a log in fixed positions; a following kernel applies them, so that all
// lookups of the step precede all of its updates.
//
// ocm_update_kernel: pre-aggregates duplicate keys of up to 1024 log entries in an LDS table, then
// issues one compare-and-swap update per distinct key, so a skewed stream (a few hot pairs) does not
// serialise on a handful of global slots.
#include "csd_internal.h"

namespace csd {
namespace {

constexpr double kLog2eF32 = (double)1.4426950408889634f;   // the fp32 constant the row-stream kernel multiplies by

__device__ __forceinline__ uint64_t slot_key(uint64_t s) { return s & CSD_OCM_KEY_MASK; }
__device__ __forceinline__ uint32_t slot_count(uint64_t s) { return (uint32_t)(s >> CSD_OCM_KEY_BITS); }

// Fibonacci hashing of the 40-bit key to a slot index; capacity is a power of two.
__device__ __forceinline__ uint64_t home_slot(uint64_t key, uint64_t capacity) {
    const uint64_t h = key * 0x9E3779B97F4A7C15ull;
    return (h >> 20) & (capacity - 1);
}

// T[key], 0 if absent.  Linear probing; an empty slot ends the search (there is no deletion).
__device__ uint32_t ocm_lookup(const uint64_t *__restrict__ ocm, uint64_t capacity, uint64_t key) {
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

// T[key] += w (saturating), inserting the key if absent.  Returns false when the table is full.
__device__ bool ocm_add(uint64_t *ocm, uint64_t capacity, uint64_t key, uint32_t w) {
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

__device__ __forceinline__ float load_logit(const void *logits, int dtype, int64_t elem) {
    if (dtype == CSD_DTYPE_F32) return ((const float *)logits)[elem];
    return __uint_as_float((uint32_t)((const uint16_t *)logits)[elem] << 16);
}

constexpr int kEpiWaves = 4;

__global__ __launch_bounds__(kEpiWaves *kWaveSize) void epilogue_kernel(EpilogueArgs a) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int b = blockIdx.x * kEpiWaves + (threadIdx.x >> 6);
    if (b >= a.B) return;                       // whole wave leaves together
    const int k = a.k, K1 = a.k + 1;
    const bool has_row = lane < K1;
    const bool is_pos = lane < k;
    const int64_t row = (int64_t)b * K1 + (has_row ? lane : 0);

    // ---- 1. combine the partials of this lane's row
    const RowPartial *pp = a.partials + row * a.partials_per_row;
    float m = -INFINITY;
    for (int j = 0; j < a.partials_per_row; ++j) m = fmaxf(m, pp[j].m);
    int t = 0x7fffffff;
    double S = 0.0;
    const double mref = (double)m * kLog2eF32;
    for (int j = 0; j < a.partials_per_row; ++j) {
        const RowPartial q = pp[j];
        if (q.m == m && q.idx < t) t = q.idx;
        if (q.s != 0.f) S += (double)q.s * exp2((double)q.cref - mref);
    }
    if (has_row) {
        a.argmax[row] = t;
        if (a.row_max) a.row_max[row] = m;
        if (a.row_sumexp) a.row_sumexp[row] = (float)S;
    }

    // ---- 2. draft token: ratio and probability
    int d = -1;
    bool valid = false;
    double ratio = 0.0;
    if (is_pos) {
        d = a.draft[(int64_t)b * k + lane];
        valid = (d >= 0) && (d < a.V);
        if (valid) {
            const float zd = load_logit(a.logits, a.dtype, row * a.row_stride + d);
            ratio = exp((double)zd - (double)m);
        }
        const int64_t o = (int64_t)b * k + lane;
        if (a.ratio) a.ratio[o] = (float)ratio;
        if (a.p_draft) a.p_draft[o] = (float)(ratio / S);
    }

    // ---- 3. match / memory lookup / gate
    const bool match = is_pos && (d == t);
    const bool diverges = is_pos && valid && !match;
    const uint64_t key = CSD_OCM_KEY((uint32_t)(diverges ? d : 0), (uint32_t)(diverges ? t : 0));
    bool is_freq = false;
    if (diverges && a.ocm != nullptr) {
        // lambda == 0 makes every pair frequent without touching the table
        is_freq = (a.lambda == 0) ? true : (ocm_lookup(a.ocm, a.capacity, key) >= a.lambda);
    }
    const bool is_safe = diverges && (ratio >= (double)a.tau);
    const bool ok = match || (is_freq && is_safe);

    // ---- 4. accepted prefix, emitted token, divergences to count
    const uint64_t fail = __builtin_amdgcn_ballot_w64(is_pos && !ok) | (1ull << k);
    const int n = (int)__builtin_ctzll(fail);                  // first failing position, k if none
    const bool processed = is_pos && (lane <= n);
    const bool counted = processed && diverges;
    const int next = __builtin_amdgcn_readlane(t, n);         // row n: stopping position or bonus row

    if (is_pos) {
        const int64_t o = (int64_t)b * k + lane;
        if (a.pos_flags) {
            uint8_t f = 0;
            if (processed) {
                if (match) f = CSD_POS_MATCH | CSD_POS_ACCEPTED;
                else if (diverges)
                    f = CSD_POS_COUNTED | (is_freq ? CSD_POS_FREQ : 0) | (is_safe ? CSD_POS_SAFE : 0) |
                        (ok ? CSD_POS_ACCEPTED : 0);
            }
            a.pos_flags[o] = f;
        }
        if (a.rej_log) a.rej_log[o] = counted ? key : CSD_OCM_EMPTY;
    }
    const uint64_t m_counted = __builtin_amdgcn_ballot_w64(counted);
    const uint64_t m_rescued = __builtin_amdgcn_ballot_w64(counted && ok);
    const uint64_t m_bad = __builtin_amdgcn_ballot_w64(processed && !valid);
    if (lane == 0) {
        a.accept_len[b] = n;
        a.next_token[b] = next;
        if (a.status) {
            if (m_bad) atomicAdd(&a.status[CSD_STATUS_BAD_DRAFT], (uint32_t)__builtin_popcountll(m_bad));
            if (m_rescued) atomicAdd(&a.status[CSD_STATUS_RESCUED], (uint32_t)__builtin_popcountll(m_rescued));
            if (m_counted) atomicAdd(&a.status[CSD_STATUS_COUNTED], (uint32_t)__builtin_popcountll(m_counted));
        }
    }
}

// ---- memory maintenance -------------------------------------------------------------------------

constexpr int kUpdThreads = 256;
constexpr int kUpdPerThread = 4;
constexpr int kUpdEntries = kUpdThreads * kUpdPerThread;   // log entries per workgroup
constexpr int kLdsSlots = 2048;                            // >= 2 * kUpdEntries: the LDS table never fills

__global__ __launch_bounds__(kUpdThreads) void ocm_update_kernel(uint64_t *ocm, uint64_t capacity,
                                                                 const uint64_t *__restrict__ keys,
                                                                 const uint32_t *__restrict__ weights, uint64_t n,
                                                                 uint32_t *status) {
    __shared__ unsigned long long lkey[kLdsSlots];
    __shared__ unsigned long long lcnt[kLdsSlots];   // 64-bit: 1024 weights of up to 2^24-1 do not wrap
    for (int i = threadIdx.x; i < kLdsSlots; i += kUpdThreads) {
        lkey[i] = CSD_OCM_EMPTY;
        lcnt[i] = 0;
    }
    __syncthreads();

    // aggregate: first thread to claim an LDS slot owns the key; counts add up (saturating later)
    const uint64_t base = (uint64_t)blockIdx.x * kUpdEntries;
    for (int j = 0; j < kUpdPerThread; ++j) {
        const uint64_t e = base + (uint64_t)j * kUpdThreads + threadIdx.x;
        if (e >= n) break;
        const uint64_t key = keys[e] & CSD_OCM_KEY_MASK;
        uint32_t w = weights ? weights[e] : 1u;
        if (key == CSD_OCM_EMPTY || w == 0) continue;
        if (w > CSD_OCM_COUNT_MAX) w = CSD_OCM_COUNT_MAX;
        uint32_t i = (uint32_t)((key * 0x9E3779B97F4A7C15ull) >> 40) & (kLdsSlots - 1);
        for (;;) {
            unsigned long long cur = lkey[i];
            if (cur == CSD_OCM_EMPTY) cur = atomicCAS(&lkey[i], (unsigned long long)CSD_OCM_EMPTY, (unsigned long long)key);
            if (cur == CSD_OCM_EMPTY || cur == key) {
                atomicAdd(&lcnt[i], (unsigned long long)w);
                break;
            }
            i = (i + 1) & (kLdsSlots - 1);
        }
    }
    __syncthreads();

    // flush: one global update per distinct key of this workgroup
    for (int i = threadIdx.x; i < kLdsSlots; i += kUpdThreads) {
        const unsigned long long key = lkey[i];
        if (key == CSD_OCM_EMPTY) continue;
        const unsigned long long sum = lcnt[i];
        const uint32_t w = (sum > CSD_OCM_COUNT_MAX) ? CSD_OCM_COUNT_MAX : (uint32_t)sum;
        if (!ocm_add(ocm, capacity, key, w) && status) atomicAdd(&status[CSD_STATUS_DROPPED], w);
    }
}

__global__ void ocm_reset_kernel(uint64_t *ocm, uint64_t capacity) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < capacity; i += stride) ocm[i] = CSD_OCM_EMPTY;
}

__global__ void ocm_lookup_kernel(const uint64_t *__restrict__ ocm, uint64_t capacity, const uint64_t *__restrict__ keys,
                                  uint32_t *__restrict__ counts, uint64_t n) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint64_t key = keys[i] & CSD_OCM_KEY_MASK;
        counts[i] = (key == CSD_OCM_EMPTY) ? 0u : ocm_lookup(ocm, capacity, key);
    }
}

}  // namespace

hipError_t launch_epilogue(const EpilogueArgs &a, hipStream_t stream) {
    if (a.B == 0) return hipSuccess;
    const dim3 grid((unsigned)((a.B + kEpiWaves - 1) / kEpiWaves));
    hipLaunchKernelGGL(epilogue_kernel, grid, dim3(kEpiWaves * kWaveSize), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_ocm_update(uint64_t *ocm, uint64_t capacity, const uint64_t *keys, const uint32_t *weights, uint64_t n,
                             uint32_t *status, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + kUpdEntries - 1) / kUpdEntries;
    hipLaunchKernelGGL(ocm_update_kernel, dim3((unsigned)blocks), dim3(kUpdThreads), 0, stream, ocm, capacity, keys, weights, n,
                       status);
    return hipGetLastError();
}

hipError_t launch_ocm_reset(uint64_t *ocm, uint64_t capacity, hipStream_t stream) {
    uint64_t blocks = (capacity + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(ocm_reset_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, ocm, capacity);
    return hipGetLastError();
}

hipError_t launch_ocm_lookup(const uint64_t *ocm, uint64_t capacity, const uint64_t *keys, uint32_t *counts, uint64_t n,
                             hipStream_t stream) {
    if (n == 0) return hipSuccess;
    uint64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(ocm_lookup_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, ocm, capacity, keys, counts, n);
    return hipGetLastError();
}

}  // namespace csd
