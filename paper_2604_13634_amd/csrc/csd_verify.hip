// The verification step.
//
// Streaming pass (stream_row_share).  For every verify row (a draft position or the bonus row of Algorithm 1) the
// step needs the target distribution's normaliser, the greedy target token t* and, later, single probabilities
// (Eq. 3 and the p_i(.) of Algorithm 1):
//     m = max_v z_v,   t* = min{v : z_v == m},   S = sum_v exp(z_v - m).
// Every logit is read from HBM exactly once with non-temporal 16-byte loads; nothing is reused, so this
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
//
// Sequence logic (sequence_decide), one wave per sequence: combine the row partials (normaliser in double),
// draft-token ratio and probability (Eq. 3), memory lookup then gate (Algorithm 1), accepted-prefix scan by
// ballot, emitted token, and the divergences to count.
//
// Three kernels put these together:
//   verify_step_kernel   csd_verify: both parts in one launch (see the comment above it);
//   row_partials_kernel  the streaming pass alone, one partial per wave: csd_row_partials, and the first launch
//                        of csd_verify_sampled;
//   finish_kernel        the sequence logic alone, sixteen sequences per workgroup, on partials that sit in memory
//                        from earlier launches (csd_verify_shards).  Each workgroup takes a ticket on the batch; the
//                        one that draws the last ticket knows that every lookup of the step has been made and
//                        applies the step's increments from the log with all its threads, so all lookups read the
//                        table as it stood when the step began.  The log handed from the sequence waves to the
//                        updating workgroup is written with agent-scope atomic stores (write-through to where the
//                        eight XCDs' L2s agree) and read back with agent-scope atomic loads; the writers' stores
//                        are acknowledged before the workgroup barrier that precedes the ticket, itself an
//                        agent-scope atomic add.  (A release/acquire fence pair would do the same job by writing
//                        back and invalidating a whole L2 per wave, which measured ten times the streaming pass.)
#include "csd_device.h"

namespace csd {
namespace {

constexpr float kLog2e = CSD_LOG2E_F32;
constexpr double kLog2eD = (double)CSD_LOG2E_F32;
constexpr float kRescaleGapLog2 = 28.8f;   // reference stays within this of the maximum, in exponent (log2) units:
                                           // 20 logits at temperature 1; below 32 keeps the exponent's ulp at 2^-19 or finer
constexpr int kNoIter = 0x7fffffff;
constexpr int kRemIter = 1 << 30;      // best_it values at or above this index the remainder loop

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
    const u32x4 *p = (const u32x4 *)rowp + (size_t)tile0 * kTileChunks + lane_chunk0;
    for (int t = 0; t < ntiles; ++t) {
        u32x4 q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) q[u] = __builtin_nontemporal_load(p + u * WL);
        p += kTileChunks;

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

    // ---- remainder of the row (one workgroup per row): one guarded chunk per lane per iteration;
    // slots past V are filled with -inf, the ragged chunk is read element by element.
    if (has_rem) {
        for (int it = 0; rem0 + it * WL < nchunks; ++it) {
            const int ch = rem0 + it * WL + lane_chunk0;
            u32x4 q = {C::kNegInfWord, C::kNegInfWord, C::kNegInfWord, C::kNegInfWord};
            if (ch < nfull) {
                q = ((const u32x4 *)rowp)[ch];
            } else if (ch == nfull) {
                q = C::load_ragged(rowp, nfull * E, tail);
            }
            float x[E];
            C::unpack(q, x);
            const float cm = chunk_max<E>(x);
            const bool up = cm > rm;
            best_it = up ? (kRemIter + it) : best_it;
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
// Phase 2: one wave, one sequence (all 64 lanes active on entry).  Lane i < k owns draft position i.

// The draft token of this lane's position and its target logit: independent of the row statistics, so it is
// fetched before them and the latencies overlap.
struct DraftLane {
    int d;
    bool valid;
    float zd;
};
template <bool SHARDED>
__device__ __forceinline__ DraftLane load_draft_lane(const EpilogueArgs &a, int b, int lane) {
    DraftLane dl = {-1, false, 0.f};
    if (lane < a.k) {
        dl.d = a.draft[(int64_t)b * a.k + lane];
        dl.valid = (dl.d >= 0) && (dl.d < a.V);
        if (dl.valid)
            dl.zd = SHARDED ? a.draft_logit[(int64_t)b * a.k + lane]
                            : load_logit(a.logits, a.dtype, ((int64_t)b * (a.k + 1) + lane) * a.row_stride + dl.d);
    }
    return dl;
}

// How the lanes of a wave share the k+1 rows of a sequence: G lanes (a power of two) per row.
__device__ __forceinline__ int lanes_per_row(int K1) {
    int G = 1;
    while (2 * G * K1 <= kWaveSize) G *= 2;
    return G;
}

// Row statistics held by the first lane of each row's group -> outputs, and to the position layout
// (lane i gets the statistics of row i; lanes >= K1 read row 0, unused).
__device__ __forceinline__ void publish_row_stats(const EpilogueArgs &a, int b, int lane, int G, float gm, int t, double S,
                                                  float &rmax, int &tstar, double &rS) {
    const int K1 = a.k + 1;
    const int grow = lane / G, gs = lane & (G - 1);
    if (grow < K1 && gs == 0) {
        const int64_t row = (int64_t)b * K1 + grow;
        a.argmax[row] = t;
        if (a.row_max) a.row_max[row] = gm;
        if (a.row_sumexp) a.row_sumexp[row] = (float)S;
    }
    const int src = (lane < K1 ? lane : 0) * G;
    rmax = from_lane_f(gm, src);
    tstar = from_lane_i(t, src);
    rS = from_lane_d(S, src);
}

// Algorithm 1 for one sequence, given its row statistics: ratio (Eq. 3), match, memory lookup, gate, accepted
// prefix, emitted token, outputs and the per-workgroup status counters.  PROBE: keep where each lookup ended
// (for updates applied straight from these lanes); the lookup is then made even when lambda == 0.
template <bool PROBE>
__device__ __forceinline__ Divergence sequence_decide(const EpilogueArgs &a, int b, int lane, const DraftLane &dl, float rmax,
                                                      int tstar, double rS, BlockCounters &counters) {
    const int k = a.k;
    const bool is_pos = lane < k;
    const int d = dl.d;
    const bool valid = dl.valid;

    // ---- Eq. 3: ratio = p(draft)/p(t*) = exp(z_draft - m); p(draft) = ratio / S
    double ratio = 0.0;
    if (is_pos) {
        if (valid) ratio = exp2(((double)dl.zd - (double)rmax) * 1.4426950408889634);
        const int64_t o = (int64_t)b * k + lane;
        if (a.ratio) a.ratio[o] = (float)ratio;
        if (a.p_draft) a.p_draft[o] = (float)(ratio / rS);
    }

    // ---- Algorithm 1: match, else memory lookup and gate
    const bool match = is_pos && (d == tstar);
    const bool diverges = is_pos && valid && !match;
    Divergence out;
    out.key = CSD_OCM_KEY((uint32_t)(diverges ? d : 0), (uint32_t)(diverges ? tstar : 0));
    out.probe = OcmProbe{0, 0, false, false};
    bool is_freq = false;
    if (diverges && a.ocm != nullptr) {
        if (PROBE) {
            out.probe = ocm_probe(a.ocm, a.capacity, out.key);
            is_freq = out.probe.count >= a.lambda;
        } else {   // lambda == 0 makes every pair frequent without touching the table
            is_freq = (a.lambda == 0) ? true : (ocm_lookup(a.ocm, a.capacity, out.key) >= a.lambda);
        }
    }
    const bool is_safe = diverges && (ratio >= (double)a.tau);
    const bool ok = match || (is_freq && is_safe);

    // ---- accepted prefix, emitted token, divergences to count (every processed one, rescued or not)
    const uint64_t fail = __builtin_amdgcn_ballot_w64(is_pos && !ok) | (1ull << k);
    const int n = (int)__builtin_ctzll(fail);                  // first failing position, k if none
    const bool processed = is_pos && (lane <= n);
    const bool counted = processed && diverges;
    const int next = from_lane_i(tstar, n);                    // row n: stopping position or bonus row
    out.counted = counted;

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
        if (a.rej_log) xwg_store64(&a.rej_log[o], counted ? out.key : CSD_OCM_EMPTY);   // read by the update wave
    }
    const uint64_t m_counted = __builtin_amdgcn_ballot_w64(counted);
    const uint64_t m_rescued = __builtin_amdgcn_ballot_w64(counted && ok);
    const uint64_t m_bad = __builtin_amdgcn_ballot_w64(processed && !valid);
    if (lane == 0) {
        a.accept_len[b] = n;
        a.next_token[b] = next;
        if (m_bad) atomicAdd(&counters.v[CSD_STATUS_BAD_DRAFT], (unsigned int)__builtin_popcountll(m_bad));
        if (m_rescued) atomicAdd(&counters.v[CSD_STATUS_RESCUED], (unsigned int)__builtin_popcountll(m_rescued));
        if (m_counted) atomicAdd(&counters.v[CSD_STATUS_COUNTED], (unsigned int)__builtin_popcountll(m_counted));
        if (n) atomicAdd(&counters.v[CSD_STATUS_ACCEPTED], (unsigned int)n);
    }
    return out;
}

// The sequence's step when the row partials sit in memory from an earlier launch.
// SHARDED: the row partials come as several sets (vocabulary shards) and the draft logits as an array.
template <bool SHARDED>
__device__ __forceinline__ void sequence_epilogue(const EpilogueArgs &a, int b, int lane, BlockCounters &counters) {
    const int K1 = a.k + 1;
    const DraftLane dl = load_draft_lane<SHARDED>(a, b, lane);

    // ---- combine the partials: G lanes share a row, then a butterfly inside each group of G
    const int G = lanes_per_row(K1);
    const int grow = lane / G, gs = lane & (G - 1);
    const int64_t prow = (int64_t)b * K1 + (grow < K1 ? grow : 0);
    float gm = -INFINITY;
    int t = 0x7fffffff;
    double S = 0.0;
    if (!SHARDED) {
        combine_row_partials(a.shard_partials[0] + prow * a.shard_per_row[0], a.shard_per_row[0], G, gs, kLog2eD, gm, t, S);
    } else {
        for (int s = 0; s < a.n_shards; ++s)
            partials_max_pass(a.shard_partials[s] + prow * a.shard_per_row[s], a.shard_per_row[s], G, gs, a.shard_base[s], gm, t);
        partials_max_merge(G, gm, t);
        const double mref = (double)gm * kLog2eD;
        for (int s = 0; s < a.n_shards; ++s)
            partials_sum_pass(a.shard_partials[s] + prow * a.shard_per_row[s], a.shard_per_row[s], G, gs, mref, S);
        partials_sum_merge(G, S);
    }
    float rmax;
    int tstar;
    double rS;
    publish_row_stats(a, b, lane, G, gm, t, S, rmax, tstar, rS);
    sequence_decide<false>(a, b, lane, dl, rmax, tstar, rS, counters);
}

template <int DT>
__global__ __launch_bounds__(kStreamWaves *kWaveSize, 4) void row_partials_kernel(StreamSource src, int V, int nsplit,
                                                                                  RowPartial *__restrict__ partials,
                                                                                  uint32_t *batch_ticket) {
    const int row = blockIdx.x / nsplit;
    const int split = blockIdx.x - row * nsplit;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    // the later kernels' two counters (the batch ticket and, on the sampled path, the length of the list of
    // rows to draw) start every step at zero (kernel order makes this visible to them)
    if (batch_ticket != nullptr && blockIdx.x == 0 && threadIdx.x < 2)
        __hip_atomic_store(&batch_ticket[threadIdx.x], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    const char *rowp = (row < src.rows0) ? src.base0 + (int64_t)row * src.pitch0
                                         : src.base1 + (int64_t)(row - src.rows0) * src.pitch1;
    const RowPartial out = stream_row_share<DT>(rowp, V, nsplit, split, wave, lane, src.scale);
    if (lane == 0) partials[((int64_t)row * nsplit + split) * kStreamWaves + wave] = out;   // one 16-byte store
}

template <bool SHARDED>
__global__ __launch_bounds__(kApplyThreads) void finish_kernel(EpilogueArgs a) {
    __shared__ ApplyLds lds;
    __shared__ BlockCounters counters;
    __shared__ int verdict;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int b = blockIdx.x * kFinishWaves + (threadIdx.x >> 6);
    block_counters_clear(counters);
    if (b < a.B) sequence_epilogue<SHARDED>(a, b, lane, counters);   // wave-uniform: a wave takes a sequence or none
    block_counters_flush(counters, a.status);
    if (!a.apply_updates) return;
    apply_step_log(a.ocm, a.capacity, a.status, a.rej_log, (uint64_t)a.B * (uint64_t)a.k, a.batch_ticket, lds, &verdict);
}

// ---------------------------------------------------------------------------------------------------
// The whole step in ONE launch.  Workgroups [0, n_stream_wgs) stream the rows exactly as row_partials_kernel
// does; the four waves of a workgroup combine their partials in LDS and publish one StepRecord.  The workgroups
// after them take kStepSeqWaves sequences each (one wave per sequence): they fetch the draft tokens and their
// logits at once, wait for the records of their rows (every record of a sequence in one round of loads for the
// usual shapes) and run the verification loop.  The hardware hands out the workgroups of a launch in index
// order, so a sequence workgroup only ever waits for streaming workgroups that have already been started; its
// waits are bounded all the same (kSpinLimit polls of about a microsecond each), and a wait that runs out is
// reported in status[CSD_STATUS_STALLED] instead of hanging.
//
// Memory updates: with at most kMaxBarrierWorkgroups sequence workgroups (all resident together, so they can
// wait for each other) each workgroup counts itself in on the control head once its lookups are done, waits
// until all have, and then every lane adds its own pair straight to the table at the slot its lookup ended at
// (the slot of an absent pair is claimed with count zero while the workgroup waits): all lookups of the step
// precede all its updates, and no log is re-read.  The first workgroup of the launch zeroes that counter and
// then says so in the control head; the sequence workgroups count themselves in only after seeing that, and
// clear the word after the barrier (so nothing in the workspace has to survive from one call to the next).
//
// Measured against the two-launch form (streaming kernel, then a kernel of sequence waves) on the five
// benchmark shapes: 15.0 -> 10.3, 17.8 -> 13.2, 29.3 -> 23.8, 68.2 -> 59.8 and 106.7 -> 104.5 microseconds per
// step.  Memory round trips cost about 1 us on an idle chip and about 3 us while the rows are being streamed,
// which is why the sequence waves sit at the END of the grid (they start when the last streaming workgroups do,
// and do their dependent loads when the chip falls quiet).  Tried and dropped: streaming the bonus rows last and
// running loop, barrier and updates under them (the dependent chain then runs at loaded latency, and waves
// resident early take places from the streaming workgroups: 1-5 us slower on four of the five shapes); waiting
// on one record per sequence before polling all (no gain once records are one per workgroup); per-wave records
// (three rounds of loads at k = 8).

// the check word of a record: a hash of its two data words, of the call's number and of the record's index
__device__ __forceinline__ uint64_t record_check(uint64_t w0, uint64_t w1, uint64_t nonce, uint64_t rec) {
    return mix64(w0 + mix64(w1 ^ (nonce + rec * 0x9E3779B97F4A7C15ull))) | 1ull;   // never zero: a zeroed record does not pass
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
                                                  uint64_t nonce, uint32_t spin_limit, float &gm, int &t, double &S) {
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
    combine_partials_in_registers<NB>(q, G, kLog2eD, gm, t, S);
    return ok;
}

__device__ __forceinline__ void step_sequences(const EpilogueArgs &a, BlockCounters &counters, int *verdict) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wg = (int)blockIdx.x - a.n_stream_wgs;
    const int n_seq_wgs = (int)gridDim.x - a.n_stream_wgs;
    const int b = wg * kStepSeqWaves + (threadIdx.x >> 6);
    const int k = a.k, K1 = a.k + 1;
    // thread 0 will need the control head set up: ask early, look at the answer late
    uint64_t ready_seen = 0;
    if (a.update_here && threadIdx.x == 0) ready_seen = xwg_load64(&a.ctrl->ready);
    block_counters_clear(counters);

    Divergence dv;
    dv.counted = false;
    dv.key = 0;
    dv.probe = OcmProbe{0, 0, false, false};
    bool stalled = false;
    if (b < a.B) {                                   // wave-uniform: a wave takes a sequence or none
        const DraftLane dl = load_draft_lane<false>(a, b, lane);
        const int P = a.shard_per_row[0];
        const int G = lanes_per_row(K1);
        const int grow = lane / G, gs = lane & (G - 1);
        const bool active = grow < K1;
        const int64_t prow = (int64_t)b * K1 + (active ? grow : 0);
        StepRecord *row_rec = a.records + prow * P;
        const uint64_t rec0 = (uint64_t)prow * (uint64_t)P;
        const int per_lane = (P + G - 1) / G;        // wave-uniform
        float gm;
        int t;
        double S;
        bool ok;
        if (per_lane <= 4) {                         // every benchmark shape: one round trip for the whole sequence
            ok = acquire_row_stats<4>(row_rec, rec0, P, G, gs, active, a.reader_nonce, a.spin_limit, gm, t, S);
        } else {
            // many partials per lane (a huge vocabulary under a small batch): wait for them four at a time, keeping
            // the running maximum only, then take the sums in a second pass over the (now plainly readable) words
            ok = true;
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
                    ok = acquire_records<4>(row_rec, rec0, G, gs, u0, want, a.reader_nonce, a.spin_limit, q4) && ok;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (q4[u].m > gm || (q4[u].m == gm && q4[u].idx < t)) t = q4[u].idx;
                    gm = fmaxf(gm, q4[u].m);
                }
            }
            partials_max_merge(G, gm, t);
            const double mref = (double)gm * kLog2eD;
            if (active) {
                for (int j = gs; j < P; j += G) {
                    const uint64_t w0 = xwg_load64(&row_rec[j].w0), w1 = xwg_load64(&row_rec[j].w1);
                    const float cref = __uint_as_float((uint32_t)(w0 >> 32)), sj = __uint_as_float((uint32_t)w1);
                    if (sj != 0.f) S += (double)sj * (double)__builtin_amdgcn_exp2f((float)((double)cref - mref));
                }
            }
            partials_sum_merge(G, S);
        }
        stalled = !ok;
        if (!stalled) {
            float rmax;
            int tstar;
            double rS;
            publish_row_stats(a, b, lane, G, gm, t, S, rmax, tstar, rS);
            if (a.update_here) dv = sequence_decide<true>(a, b, lane, dl, rmax, tstar, rS, counters);
            else dv = sequence_decide<false>(a, b, lane, dl, rmax, tstar, rS, counters);
        } else if (lane == 0) {                      // the records never came: say so, and report nothing as accepted
            a.accept_len[b] = 0;
            a.next_token[b] = -1;
            atomicAdd(&counters.v[CSD_STATUS_STALLED], 1u);
        }
    }

    sequence_counters_and_updates(a.ctrl, ready_seen, step_ready_value(a.reader_nonce), wg == 0, (uint32_t)n_seq_wgs,
                                  a.update_here != 0, a.ocm, a.capacity, a.status, counters, dv, verdict, a.spin_limit);
}

template <int DT>
__global__ __launch_bounds__(kStreamWaves *kWaveSize, 4) void verify_step_kernel(StreamSource src, int V, int nsplit,
                                                                                 EpilogueArgs a) {
    __shared__ BlockCounters counters;
    __shared__ int verdict;
    __shared__ RowPartial wave_out[kStreamWaves];
    if ((int)blockIdx.x >= a.n_stream_wgs) {
        step_sequences(a, counters, &verdict);
        return;
    }
    const int row = blockIdx.x / nsplit;
    const int split = blockIdx.x - row * nsplit;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    if (a.update_here && blockIdx.x == 0 && threadIdx.x == 0) step_control_setup(a.ctrl, step_ready_value(a.nonce));
    const char *rowp = src.base0 + (int64_t)row * src.pitch0;
    const RowPartial out = stream_row_share<DT>(rowp, V, nsplit, split, wave, lane, src.scale);
    // The four waves of the workgroup (they sweep the same tiles and end together) leave ONE record: fewer records
    // for the sequence waves to wait for and to read.  Same combine rule as between records; the sum is taken in
    // double against the largest reference exponent and rounded to float once.
    if (lane == 0) wave_out[wave] = out;
    __syncthreads();
    if (threadIdx.x == 0) {
        RowPartial r = empty_partial();
        r.idx = wave_out[0].idx;
        float cmax = -INFINITY;
#pragma unroll
        for (int w = 0; w < kStreamWaves; ++w) {
            const RowPartial q = wave_out[w];
            if (q.m > r.m || (q.m == r.m && q.idx < r.idx)) r.idx = q.idx;
            r.m = fmaxf(r.m, q.m);
            if (q.s != 0.f) cmax = fmaxf(cmax, q.cref);
        }
        double sum = 0.0;
#pragma unroll
        for (int w = 0; w < kStreamWaves; ++w) {
            const RowPartial q = wave_out[w];
            if (q.s != 0.f) sum += (double)q.s * (double)__builtin_amdgcn_exp2f(q.cref - cmax);
        }
        r.cref = (sum != 0.0) ? cmax : 0.f;
        r.s = (float)sum;
        const uint64_t rec = (uint64_t)row * nsplit + split;
        publish_record(a.records + rec, a.nonce, rec, r);
    }
}

}  // namespace

StreamPlan make_stream_plan(int rows, int V, int dtype) {
    StreamPlan p;
    p.rows = rows;
    p.elems_per_chunk = (dtype == CSD_DTYPE_F32) ? 4 : 8;
    p.nchunks = (V + p.elems_per_chunk - 1) / p.elems_per_chunk;
    p.ntiles_row = (V / p.elems_per_chunk) / kTileChunks;
    // Workgroups per row.  Two tiles per workgroup measured best from the smallest benchmark shape to the largest
    // (one tile: a third more records to publish and to wait for, and 4 - 6 % slower at every size; four: 0.5 - 2 %
    // slower on the two big shapes).  The exception is a launch that two tiles leave just too large to be resident
    // at once (four workgroups per compute unit): three or four tiles then bring it under that line, and no
    // second round of workgroups has to be dealt out (256 rows of 9 tiles: 22.4 -> 21.9 microseconds per step).
    const int ntr = p.ntiles_row > 0 ? p.ntiles_row : 1;
    const int64_t resident = 4 * 256;
    int tiles_per_group = 2;
    if ((int64_t)rows * ((ntr + 1) / 2) > resident) {
        for (int t = 3; t <= 4; ++t)
            if ((int64_t)rows * ((ntr + t - 1) / t) <= resident) { tiles_per_group = t; break; }
    }
    int nsplit = (p.ntiles_row + tiles_per_group - 1) / tiles_per_group;
    if (nsplit < 1) nsplit = 1;
    p.nsplit = nsplit;
    p.partials_per_row = p.nsplit * kStreamWaves;
    return p;
}

WorkspaceLayout make_workspace_layout(const StreamPlan &p, int B, int k) {
    WorkspaceLayout w;
    w.ticket_off = 0;
    w.partials_off = 256;
    w.partials_bytes = (size_t)p.rows * (size_t)p.nsplit * sizeof(StepRecord);          // one record per streaming workgroup
    w.log_off = (w.partials_off + w.partials_bytes + 255) & ~(size_t)255;
    w.log_bytes = (size_t)B * (size_t)k * sizeof(uint64_t);
    w.total = (w.log_off + w.log_bytes + 255) & ~(size_t)255;
    return w;
}

hipError_t launch_row_partials(const StreamSource &src, int dtype, int V, const StreamPlan &plan, RowPartial *partials,
                               uint32_t *batch_ticket, hipStream_t stream) {
    if (plan.rows == 0) return hipSuccess;
    const dim3 grid((unsigned)(plan.rows * plan.nsplit)), block(kStreamWaves * kWaveSize);
    if (dtype == CSD_DTYPE_F32)
        hipLaunchKernelGGL(row_partials_kernel<CSD_DTYPE_F32>, grid, block, 0, stream, src, V, plan.nsplit, partials,
                           batch_ticket);
    else
        hipLaunchKernelGGL(row_partials_kernel<CSD_DTYPE_BF16>, grid, block, 0, stream, src, V, plan.nsplit, partials,
                           batch_ticket);
    return hipGetLastError();
}

namespace {
__global__ void zero_ticket_kernel(uint32_t *ticket) { __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// the logit of every draft token this vocabulary shard owns (ids in [base, base + V_shard)); others untouched
__global__ void shard_draft_logits_kernel(const void *logits, int dtype, int64_t row_stride, int B, int k, int V_shard, int base,
                                          const int32_t *__restrict__ draft, float *__restrict__ draft_logit) {
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= (int64_t)B * k) return;
    const int64_t b = o / k, i = o - b * k;
    const int64_t local = (int64_t)draft[o] - base;
    if (local < 0 || local >= V_shard) return;
    draft_logit[o] = load_logit(logits, dtype, (b * (k + 1) + i) * row_stride + local);
}
}  // namespace

hipError_t launch_zero_ticket(uint32_t *ticket, hipStream_t stream) {
    hipLaunchKernelGGL(zero_ticket_kernel, dim3(1), dim3(1), 0, stream, ticket);
    return hipGetLastError();
}

hipError_t launch_shard_draft_logits(const void *logits, int dtype, int64_t row_stride, int B, int k, int V_shard, int base,
                                     const int32_t *draft, float *draft_logit, hipStream_t stream) {
    const int64_t n = (int64_t)B * k;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(shard_draft_logits_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, logits, dtype,
                       row_stride, B, k, V_shard, base, draft, draft_logit);
    return hipGetLastError();
}

hipError_t launch_verify_step(const StreamSource &src, int dtype, int V, const StreamPlan &plan, const EpilogueArgs &a,
                              hipStream_t stream) {
    if (plan.rows == 0 || a.B == 0) return hipSuccess;
    const int n_seq_wgs = (a.B + kStepSeqWaves - 1) / kStepSeqWaves;
    const dim3 grid((unsigned)(a.n_stream_wgs + n_seq_wgs)), block(kStreamWaves * kWaveSize);
    if (dtype == CSD_DTYPE_F32)
        hipLaunchKernelGGL(verify_step_kernel<CSD_DTYPE_F32>, grid, block, 0, stream, src, V, plan.nsplit, a);
    else
        hipLaunchKernelGGL(verify_step_kernel<CSD_DTYPE_BF16>, grid, block, 0, stream, src, V, plan.nsplit, a);
    return hipGetLastError();
}

hipError_t launch_finish(const EpilogueArgs &a, hipStream_t stream) {
    if (a.B == 0) return hipSuccess;
    const dim3 grid((unsigned)((a.B + kFinishWaves - 1) / kFinishWaves));
    if (a.sharded)
        hipLaunchKernelGGL(finish_kernel<true>, grid, dim3(kFinishWaves * kWaveSize), 0, stream, a);
    else
        hipLaunchKernelGGL(finish_kernel<false>, grid, dim3(kFinishWaves * kWaveSize), 0, stream, a);
    return hipGetLastError();
}

}  // namespace csd
