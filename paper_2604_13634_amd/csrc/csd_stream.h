// The streaming pass over one row share, and the records by which streaming workgroups hand their results to
// waves of the same launch.  Shared by the greedy step (csd_verify.hip) and the first launch of the sampled step
// (csd_sampled.hip).
//
// Streaming pass (stream_row_share).  For every verify row (a draft position or the bonus row of Algorithm 1) the
// step needs the target distribution's normaliser, the greedy target token t* and, later, single probabilities
// (Eq. 3 and the p_i(.) of Algorithm 1):
//     m = max_v z_v,   t* = min{v : z_v == m},   S = sum_v exp(z_v - m).
// Every logit is read from HBM exactly once with non-temporal 16-byte loads (buffer loads for bf16); nothing is reused, so this
// pass is bound by HBM bandwidth (no MFMA, no LDS staging).  A row's 32 KiB tiles are cut into
// `nsplit` contiguous runs, one per workgroup of 4 waves (dealing the tiles round-robin to the row's workgroups
// instead measures the same); inside a tile the waves interleave 1 KiB wave-loads.
// Each wave keeps its own running state; there is no barrier and no cross-wave step inside the sweep.
//
//   Per-lane state (fp32): rm = running maximum; best_q = the 16-byte chunk at which rm last strictly
//   increased and best_it = its iteration, i.e. the first chunk of this lane that holds rm (a lane
//   visits chunks in ascending address order, so "first" is "lowest token id"); s[E] = sums of
//   2^(z*log2e - c), one per element slot of a chunk, against a WAVE-UNIFORM reference exponent c.
//   c is not the running maximum: it is only kept within kRescaleGapLog2 of it (in exponent units), which is all floating point
//   needs (no overflow, full relative precision).  A rescale (wave reduction + multiply) happens only
//   when some lane's maximum climbs more than that above the reference - at the first tile, then
//   almost never - so the steady-state loop is unpack, max3, fma, v_exp_f32, add and one compare per
//   tile.  The exponent error of a term is half an ulp of |z*log2e - c| < 32, i.e. below 7e-7 relative;
//   c itself is carried exactly into the combine.  c is a float near m*log2e, so the largest term is
//   2^d with |d| <= ulp(c)/2: this is why logits are limited to |z| <= 2^29 (d <= 32, sums stay in range).
#pragma once
#include "csd_device.h"

namespace csd {
namespace {

constexpr float kLog2e = CSD_LOG2E_F32;
constexpr double kLog2eD = (double)CSD_LOG2E_F32;
constexpr float kRescaleGapLog2 = 28.8f;   // reference stays within this of the maximum, in exponent (log2) units:
                                           // 20 logits at temperature 1; below 32 keeps the exponent's ulp at 2^-19 or finer
constexpr int kNoIter = 0x7fffffff;
constexpr int kBufferRsrcFlags = 0x00020000;   // fourth word of a raw buffer descriptor on gfx9: 32-bit data format, no swizzle
constexpr int kBufferNonTemporal = 2;          // cache-policy bits of a buffer load: the `nt` bit alone
// Which storage types sweep with buffer loads.  The bf16 sweep keeps the vector ALUs two thirds busy, and the 64-bit
// address arithmetic of global loads is vector-ALU work: buffer loads took 1.2 - 2 microseconds (1 - 2 %) off the
// largest bf16 step and put the streaming pass at the rate of a read-only kernel.  (Of the cache-policy bits only
// `nt` matters: plain, sc0, sc1 or both read 6.2 TB/s in a read-only probe, every combination with nt 6.97.)  The
// fp32 sweep has the ALUs one third busy and nothing to gain there; its step measured 0.6 microseconds slower with
// buffer loads (the streaming pass alone 0.35 faster), so it keeps the global loads.
template <int DT> constexpr bool kBufferLoads = (DT == CSD_DTYPE_BF16);
constexpr int kRemIter = 1 << 30;      // best_it values at or above this index the remainder loop

// Which share of its row a streaming workgroup takes: the workgroup's place in the row, rotated by the row when
// the number of shares is even.  Workgroups go to the eight XCDs in turn by index, and the last share of a row is
// the short one (fewest tiles plus the ragged end): with the place alone, eight shares per row would send every
// row's short share to the same XCD (four: to two of them), which then runs out of work while the others still
// stream - at 2304 rows of 8 shares the step measured 275 microseconds without the rotation, 269 with it.  An odd
// number of shares walks through the XCDs by itself (and measured 1 % slower rotated).
__device__ __forceinline__ int share_of_workgroup(int place, int row, int nsplit) {
    return (nsplit & 1) ? place : (place + row) % nsplit;
}

// ---------------------------------------------------------------------------------------------------
// Phase 1: this wave's share of one row -> one RowPartial (returned in lane-uniform registers).
template <int DT>
__device__ __forceinline__ RowPartial stream_row_share(const char *__restrict__ rowp, int V, int nsplit, int split,
                                                       int wave, int lane, float scale) {
    using C = Chunk<DT>;
    constexpr int E = C::E;
    constexpr int W = kStreamWaves;
    constexpr int U = kStreamUnroll;
    constexpr int WL = W * kWaveSize;              // chunks one load instruction of the workgroup covers

    const int nfull = V / E;                       // whole 16-byte chunks of the row
    const int tail = V - nfull * E;                // logits in the ragged last chunk
    const int nchunks = nfull + (tail ? 1 : 0);
    const int ntiles_row = nfull / kTileChunks;    // whole tiles of whole chunks
    const int rem0 = ntiles_row * kTileChunks;     // first chunk of the remainder
    // This workgroup's tiles: a contiguous run of the row (the first `extra` workgroups take one tile more); the
    // last workgroup, which has the fewest tiles, also takes the remainder.
    const int base_tiles = ntiles_row / nsplit, extra = ntiles_row - base_tiles * nsplit;
    const int tile0 = split * base_tiles + (split < extra ? split : extra);
    const int ntiles = base_tiles + (split < extra ? 1 : 0);
    const bool has_rem = (split == nsplit - 1) && (rem0 < nchunks);

    float rm = -INFINITY;      // running max of this lane
    int best_it = kNoIter;     // iteration that first reached rm ...
    u32x4 best_q = {0u, 0u, 0u, 0u};   // ... and the chunk read there
    float s[E];
#pragma unroll
    for (int j = 0; j < E; ++j) s[j] = 0.f;
    float c = 0.f;             // wave-uniform reference exponent (log2 units)
    float mth = -INFINITY;     // rescale when a lane maximum exceeds this
    const float gap = kRescaleGapLog2 / scale;   // the same distance in logit units
    const int lane_chunk0 = wave * kWaveSize + lane;

    auto rescale = [&]() {
        const float wm = wave_allreduce_f(rm, MaxF());
        const float cn = wm * scale;
        const float sc = __builtin_amdgcn_exp2f(c - cn);
#pragma unroll
        for (int j = 0; j < E; ++j) s[j] = (s[j] == 0.f) ? 0.f : s[j] * sc;
        c = cn;
        mth = wm + gap;
    };

    // ---- whole tiles: U independent non-temporal 16-byte loads per lane.
    // Local tile t is row tile tile0 + t; its chunk for (u, this lane) is
    //     (tile0 + t) * kTileChunks + u*WL + lane_chunk0   < ntiles_row * kTileChunks <= nfull.
    // bf16: buffer loads - one 32-bit offset per lane and the eight loads' strides in the instruction's scalar
    // offset; the descriptor covers the row's whole chunks, every offset below lies inside it.
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)rowp, 0, nfull * 16, kBufferRsrcFlags);
    int voff = (tile0 * kTileChunks + lane_chunk0) * 16;
    const u32x4 *p = (const u32x4 *)rowp + (size_t)tile0 * kTileChunks + lane_chunk0;
    for (int t = 0; t < ntiles; ++t) {
        u32x4 q[U];
        if constexpr (kBufferLoads<DT>) {
#pragma unroll
            for (int u = 0; u < U; ++u) q[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, u * WL * 16, kBufferNonTemporal);
            voff += kTileChunks * 16;
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) q[u] = __builtin_nontemporal_load(p + u * WL);
            p += kTileChunks;
        }

        float x[U][E];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            C::unpack(q[u], x[u]);
            const float cm = chunk_max<E>(x[u]);
            const bool up = cm > rm;
            best_it = up ? (t * U + u) : best_it;
            best_q.x = up ? q[u].x : best_q.x;
            best_q.y = up ? q[u].y : best_q.y;
            best_q.z = up ? q[u].z : best_q.z;
            best_q.w = up ? q[u].w : best_q.w;
            rm = __builtin_fmaxf(rm, cm);
        }
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(rm > mth) != 0, 0)) rescale();
        const float nc = -c;
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int j = 0; j < E; ++j) s[j] += __builtin_amdgcn_exp2f(__builtin_fmaf(x[u][j], scale, nc));
        }
    }

    // ---- remainder of the row (one workgroup per row): less than a tile of whole chunks, swept as one guarded
    // tile - same chunk for (u, lane) as in a whole tile, all loads issued before any arithmetic (taken one
    // chunk per lane at a time, this share held its place on the compute unit for five memory latencies where
    // its neighbours need two); slots past the whole chunks are filled with -inf.  Plain loads here: with
    // non-temporal ones the largest benchmark shape measured 1.7 microseconds slower (105.6 against 103.9; the
    // one-chunk-at-a-time form 105.0), the small shapes the same (11.7 against 13.1, 8.7 against 9.8 per step).
    // Then, when V is not a multiple of E, the ragged last chunk, read element by element by the one lane
    // that owns it.
    if (has_rem) {
        {
            u32x4 q[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int ch = rem0 + u * WL + lane_chunk0;
                q[u].x = q[u].y = q[u].z = q[u].w = C::kNegInfWord;
                if (ch < nfull) q[u] = ((const u32x4 *)rowp)[ch];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {             // chunk by chunk: few registers live beside the loads
                float x[E];
                C::unpack(q[u], x);
                const float cm = chunk_max<E>(x);
                const bool up = cm > rm;
                best_it = up ? (kRemIter + u) : best_it;
                best_q.x = up ? q[u].x : best_q.x;
                best_q.y = up ? q[u].y : best_q.y;
                best_q.z = up ? q[u].z : best_q.z;
                best_q.w = up ? q[u].w : best_q.w;
                rm = __builtin_fmaxf(rm, cm);
                if (__builtin_amdgcn_ballot_w64(rm > mth) != 0) rescale();
                const float nc = -c;
#pragma unroll
                for (int j = 0; j < E; ++j) s[j] += __builtin_amdgcn_exp2f(__builtin_fmaf(x[j], scale, nc));
            }
        }
        if (tail) {                                   // chunk nfull: lane (nfull - rem0) mod WL of the workgroup, at u = its quotient
            const int off = nfull - rem0 - lane_chunk0;
            const bool mine = off >= 0 && off % WL == 0;
            u32x4 q = {C::kNegInfWord, C::kNegInfWord, C::kNegInfWord, C::kNegInfWord};
            if (mine) q = C::load_ragged(rowp, nfull * E, tail);
            float x[E];
            C::unpack(q, x);
            const float cm = chunk_max<E>(x);
            const bool up = cm > rm;
            best_it = up ? (kRemIter + off / WL) : best_it;
            best_q.x = up ? q.x : best_q.x;
            best_q.y = up ? q.y : best_q.y;
            best_q.z = up ? q.z : best_q.z;
            best_q.w = up ? q.w : best_q.w;
            rm = __builtin_fmaxf(rm, cm);
            if (__builtin_amdgcn_ballot_w64(rm > mth) != 0) rescale();
            const float nc = -c;
#pragma unroll
            for (int j = 0; j < E; ++j) s[j] += __builtin_amdgcn_exp2f(__builtin_fmaf(x[j], scale, nc));
        }
    }

    // ---- wave result
    float sl = s[0];
#pragma unroll
    for (int j = 1; j < E; ++j) sl += s[j];
    const float ws = wave_allreduce_f(sl, AddF());
    const float wm = wave_allreduce_f(rm, MaxF());
    // Lanes that hold the wave maximum name the lowest token id at which they saw it: the first element
    // of their saved chunk equal to it (float compare: -0 == +0).  The wave takes the smallest.
    int my_idx = kNoIter;
    if (best_it != kNoIter && rm == wm) {
        const int chunk = (best_it >= kRemIter)
                              ? rem0 + (best_it - kRemIter) * WL + lane_chunk0
                              : (tile0 + best_it / U) * kTileChunks + (best_it % U) * WL + lane_chunk0;
        float x[E];
        C::unpack(best_q, x);
        int j0 = E - 1;
#pragma unroll
        for (int j = E - 1; j >= 0; --j) j0 = (x[j] == wm) ? j : j0;
        my_idx = chunk * E + j0;
    }
    int idx = wave_allreduce_i(my_idx, MinI());
    // a share without any finite value reports the first token it covers (token 0 if it covers nothing)
    if (idx == kNoIter) idx = ((ntiles > 0) ? tile0 * kTileChunks : (has_rem ? rem0 : 0)) * E;
    RowPartial out;
    out.m = wm;
    out.cref = c;
    out.s = ws;
    out.idx = idx;
    return out;
}

// ---------------------------------------------------------------------------------------------------
// Records: what a streaming workgroup leaves for the waves of the same launch that wait for it.

// The check word of a record: its two data words, each through a multiplication of its own (a bijection of that word,
// so a read that mixes an old word with a new one fails), keyed by the call's number and the record's index (what
// an earlier call left behind fails).  Two independent multiplications and a few shifts: the publishing workgroup
// holds its place on the compute unit while it computes this, and every reader computes it per record it polls.
__device__ __forceinline__ uint64_t record_check(uint64_t w0, uint64_t w1, uint64_t nonce, uint64_t rec) {
    const uint64_t key = nonce + rec * 0x9E3779B97F4A7C15ull;
    const uint64_t a = (w0 ^ key) * 0xBF58476D1CE4E5B9ull;
    const uint64_t b = (w1 + key) * 0x94D049BB133111EBull;
    uint64_t c = a ^ ((b << 32) | (b >> 32));
    c ^= c >> 29;
    return c ? c : 1ull;                             // never zero: a zeroed record does not pass
}
__device__ __forceinline__ void publish_record(StepRecord *r, uint64_t nonce, uint64_t rec, const RowPartial &p) {
    const uint64_t w0 = (uint64_t)__float_as_uint(p.m) | ((uint64_t)__float_as_uint(p.cref) << 32);
    const uint64_t w1 = (uint64_t)__float_as_uint(p.s) | ((uint64_t)(uint32_t)p.idx << 32);
    xwg_store64(&r->w0, w0);
    xwg_store64(&r->w1, w1);
    xwg_store64(&r->check, record_check(w0, w1, nonce, rec));
}

// Records j = gs + (u0 + u)*G, u < N, of one row: loaded until they pass, all N of a round in flight together
// (one memory round trip when they are all there).  `want` says which of them this lane needs; passing ones
// are decoded into q and their check word zeroed.  Returns false when the wait ran out.  Called by all lanes
// of the wave together.
template <int N>
__device__ __forceinline__ bool acquire_records(StepRecord *row_rec, uint64_t rec0, int G, int gs, int u0, uint32_t want,
                                                uint64_t nonce, uint32_t spin_limit, RowPartial (&q)[N]) {
    uint32_t pend = want;
    for (uint32_t spin = 0;; ++spin) {
        uint64_t w0[N], w1[N], ck[N];
#pragma unroll
        for (int u = 0; u < N; ++u) {
            if ((pend >> u) & 1u) {
                const StepRecord *r = row_rec + gs + (u0 + u) * G;
                w0[u] = xwg_load64(&r->w0);
                w1[u] = xwg_load64(&r->w1);
                ck[u] = xwg_load64(&r->check);
            }
        }
#pragma unroll
        for (int u = 0; u < N; ++u) {
            if ((pend >> u) & 1u) {
                const uint64_t j = (uint64_t)(gs + (u0 + u) * G);
                if (ck[u] == record_check(w0[u], w1[u], nonce, rec0 + j)) {
                    q[u].m = __uint_as_float((uint32_t)w0[u]);
                    q[u].cref = __uint_as_float((uint32_t)(w0[u] >> 32));
                    q[u].s = __uint_as_float((uint32_t)w1[u]);
                    q[u].idx = (int32_t)(uint32_t)(w1[u] >> 32);
                    xwg_store64(&row_rec[gs + (u0 + u) * G].check, 0ull);
                    pend &= ~(1u << u);
                }
            }
        }
        if (__builtin_amdgcn_ballot_w64(pend != 0u) == 0ull) return true;
        if (spin >= spin_limit) return false;
        __builtin_amdgcn_s_sleep(kSpinSleep);
    }
}

// All records of this lane's share of its row -> (m, t*, S) of the row, in the first lane of its group, with the
// arithmetic of the two-launch combine, in its order.
template <int NB>
__device__ __forceinline__ bool acquire_row_stats(StepRecord *row_rec, uint64_t rec0, int P, int G, int gs, bool active,
                                                  double scale, uint64_t nonce, uint32_t spin_limit, float &gm, int &t, double &S) {
    RowPartial q[NB];
    uint32_t want = 0;
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        q[u] = empty_partial();
        if (active && gs + u * G < P) want |= 1u << u;
    }
    const bool ok = acquire_records<NB>(row_rec, rec0, G, gs, 0, want, nonce, spin_limit, q);
    gm = -INFINITY;
    t = 0x7fffffff;
    S = 0.0;
    combine_partials_in_registers<NB>(q, G, scale, gm, t, S);
    return ok;
}

// The same for any number of records per row: up to four per lane take the single round above (every benchmark
// shape); more (a huge vocabulary under a small batch) are waited for four at a time, keeping the running
// maximum only, and the sums are taken in a second pass over the (now plainly readable) words.
__device__ __forceinline__ bool acquire_row_stats_any(StepRecord *row_rec, uint64_t rec0, int P, int G, int gs, bool active,
                                                      double scale, uint64_t nonce, uint32_t spin_limit, float &gm, int &t,
                                                      double &S) {
    const int per_lane = (P + G - 1) / G;            // wave-uniform
    if (per_lane <= 4) return acquire_row_stats<4>(row_rec, rec0, P, G, gs, active, scale, nonce, spin_limit, gm, t, S);
    bool ok = true;
    gm = -INFINITY;
    t = 0x7fffffff;
    S = 0.0;
    for (int u0 = 0; u0 < per_lane; u0 += 4) {
        RowPartial q4[4];
        uint32_t want = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            q4[u] = empty_partial();
            if (active && gs + (u0 + u) * G < P) want |= 1u << u;
        }
        if (__builtin_amdgcn_ballot_w64(want != 0u) != 0ull)
            ok = acquire_records<4>(row_rec, rec0, G, gs, u0, want, nonce, spin_limit, q4) && ok;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (q4[u].m > gm || (q4[u].m == gm && q4[u].idx < t)) t = q4[u].idx;
            gm = fmaxf(gm, q4[u].m);
        }
    }
    partials_max_merge(G, gm, t);
    const double mref = (double)gm * scale;
    if (active) {
        for (int j = gs; j < P; j += G) {
            const uint64_t w0 = xwg_load64(&row_rec[j].w0), w1 = xwg_load64(&row_rec[j].w1);
            const float cref = __uint_as_float((uint32_t)(w0 >> 32)), sj = __uint_as_float((uint32_t)w1);
            if (sj != 0.f) S += (double)sj * (double)__builtin_amdgcn_exp2f((float)((double)cref - mref));
        }
    }
    partials_sum_merge(G, S);
    return ok;
}

// The four waves of a streaming workgroup (they sweep the same tiles and end together) leave ONE record: fewer
// records for the waiting waves to poll and to read.  Same combine rule as between records; the sum is taken in
// double against the largest reference exponent and rounded to float once.  The workgroup keeps its place on the
// compute unit until the record has left, so this is kept short: lanes 0 - 3 of the first wave take one wave's
// partial each and combine them with two butterfly steps inside their quad (one lane's loop over the four, with a
// two-round hash behind the check word, was 190 dependent instructions; this form measured 0.2 - 0.4 microseconds
// per step faster on every benchmark shape).  Called by every thread; `wave_out` is the workgroup's LDS staging.
template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) {
    const long long b = __double_as_longlong(v);
    const int lo = dpp_i<CTRL>((int)(b & 0xFFFFFFFFll)), hi = dpp_i<CTRL>((int)(b >> 32));
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
template <int CTRL>
__device__ __forceinline__ void quad_max_step(float &m, int &idx) {   // larger m wins, equal m: smaller idx
    const float om = __int_as_float(dpp_i<CTRL>(__float_as_int(m)));
    const int oi = dpp_i<CTRL>(idx);
    if (om > m || (om == m && oi < idx)) idx = oi;
    m = fmaxf(m, om);
}
__device__ __forceinline__ void publish_workgroup_share(RowPartial (&wave_out)[kStreamWaves], const RowPartial &out, int wave,
                                                        int lane, StepRecord *records, uint64_t rec, uint64_t nonce) {
    static_assert(kStreamWaves == 4, "the combine is a butterfly inside one quad");
    if (lane == 0) wave_out[wave] = out;
    __syncthreads();
    if (threadIdx.x >= kStreamWaves) return;
    const RowPartial q = wave_out[threadIdx.x];
    float m = q.m;
    int idx = q.idx;
    quad_max_step<0xB1>(m, idx);                     // quad_perm [1,0,3,2]
    quad_max_step<0x4E>(m, idx);                     // quad_perm [2,3,0,1]
    float cmax = (q.s != 0.f) ? q.cref : -INFINITY;
    cmax = fmaxf(cmax, __int_as_float(dpp_i<0xB1>(__float_as_int(cmax))));
    cmax = fmaxf(cmax, __int_as_float(dpp_i<0x4E>(__float_as_int(cmax))));
    double sum = (q.s != 0.f) ? (double)q.s * (double)__builtin_amdgcn_exp2f(q.cref - cmax) : 0.0;
    sum += dpp_d<0xB1>(sum);
    sum += dpp_d<0x4E>(sum);
    if (threadIdx.x == 0) {
        RowPartial r;
        r.m = m;
        r.idx = idx;
        r.cref = (sum != 0.0) ? cmax : 0.f;
        r.s = (float)sum;
        publish_record(records + rec, nonce, rec, r);
    }
}

}  // namespace
}  // namespace csd
