// The verification step.
//
// Streaming pass: stream_row_share in csd_stream.h (described there), one share of one row per workgroup.
//
// Sequence logic (sequence_decide), one wave per sequence: combine the row partials (normaliser in double),
// draft-token ratio and probability (Eq. 3), memory lookup then gate (Algorithm 1), accepted-prefix scan by
// ballot, emitted token, and the divergences to count.
//
// Three kernels put these together:
//   verify_step_kernel   csd_verify: both parts in one launch (see the comment above it);
//   row_partials_kernel  the streaming pass alone, one partial per wave: csd_row_partials (the first launch of
//                        csd_verify_sampled has its own kernel around the same pass, csd_sampled.hip);
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
#include <atomic>

#include "csd_stream.h"

namespace csd {
namespace {

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

// Row statistics held by the first lane of each row's group (rows 0 .. nrows-1 of the sequence) -> outputs, and to
// the position layout (lane i gets the statistics of row i; lanes >= K1 read row 0, unused).
__device__ __forceinline__ void publish_row_stats(const EpilogueArgs &a, int b, int lane, int G, int nrows, float gm, int t,
                                                  double S, float &rmax, int &tstar, double &rS) {
    const int K1 = a.k + 1;
    const int grow = lane / G, gs = lane & (G - 1);
    if (grow < nrows && gs == 0) {
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
// bonus_known: lane k holds the bonus row's t*; without it the emitted token of a sequence that keeps all its
// draft tokens is left to whoever takes the bonus row (the loop itself never reads that row).
template <bool PROBE>
__device__ __forceinline__ Divergence sequence_decide(const EpilogueArgs &a, int b, int lane, const DraftLane &dl, float rmax,
                                                      int tstar, double rS, bool bonus_known, BlockCounters &counters) {
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
    out.n = n;

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
        if (bonus_known || n < k) a.next_token[b] = next;
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
    publish_row_stats(a, b, lane, G, K1, gm, t, S, rmax, tstar, rS);
    sequence_decide<false>(a, b, lane, dl, rmax, tstar, rS, true, counters);
}

template <int DT>
__global__ __launch_bounds__(kStreamWaves *kWaveSize, 4) void row_partials_kernel(StreamSource src, int V, int nsplit,
                                                                                  RowPartial *__restrict__ partials) {
    const int row = blockIdx.x / nsplit;
    const int split = share_of_workgroup((int)blockIdx.x - row * nsplit, row, nsplit);
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
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
// until all have, and then adds its pairs straight to the table at the slots its lookups ended at - one add per
// distinct pair of the workgroup, carrying the number of its lanes that hold the pair (the slot of an absent pair
// is claimed with count zero while the workgroup waits): all lookups of the step precede all its updates, and no
// log is re-read.  The first workgroup of the launch zeroes that counter and then says so in the control head; the
// sequence workgroups count themselves in only after seeing that, and clear the word after the barrier (so nothing
// in the workspace has to survive from one call to the next).
//
// Two grid orders (make_step_order).  Plain: rows in row order, then the sequence workgroups, which take all k+1
// rows of their sequences in one round of record loads.  Bonus rows last (launches too large to be resident at
// once): the rows of the draft positions, then the bonus rows, then the sequence workgroups, which take the draft
// positions' rows only - all the loop, the lookups, the barrier and the updates depend on - and so start before the
// stream has ended; a last set of workgroups takes the bonus rows' statistics and the emitted token of sequences
// that kept every draft token (step_bonus_rows), one round trip after the last streaming workgroup.
//
// Measured against the two-launch form (streaming kernel, then a kernel of sequence waves) on the five
// benchmark shapes: 15.0 -> 10.3, 17.8 -> 13.2, 29.3 -> 23.8, 68.2 -> 59.8 and 106.7 -> 104.5 microseconds per
// step.  Memory round trips cost about 1 us on an idle chip and 3 - 5 us while the rows are being streamed,
// which is why the sequence waves sit at the END of the grid (they start when the last streaming workgroups do,
// and do their dependent loads when the chip falls quiet).  Tried and dropped: sequence workgroups placed earlier
// in the grid (see make_step_order); waiting on one record per sequence before polling all (no gain once records
// are one per workgroup); per-wave records (three rounds of loads at k = 8).


// What a sequence's loop leaves for the wave that takes its bonus row (bonus-rows-last order): the accepted length,
// or this mark when the loop's own wait ran out.
constexpr uint64_t kSeqWordStalled = 0xFFFFFFFFull;

// A sequence workgroup: four sequences, one wave each.  wg = its number among the n_seq_wgs sequence workgroups.
// Plain order: the statistics of all k+1 rows, the loop, the emitted token.  Bonus-rows-last order: the rows of
// the draft positions only - everything the lookups, the barrier and the updates depend on - while the bonus rows
// are still being streamed; the accepted length is handed on in a published word.
__device__ __forceinline__ void step_sequences(const EpilogueArgs &a, int wg, BlockCounters &counters, StepMergeLds &merge,
                                               int *verdict) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int b = wg * kStepSeqWaves + (threadIdx.x >> 6);
    const int k = a.k, K1 = a.k + 1;
    const bool bonus_later = a.order.bonus_last != 0;
    const int nrows = bonus_later ? k : K1;          // rows whose statistics this wave takes
    // thread 0 will need the control head set up: ask early, look at the answer late
    uint64_t ready_seen = 0;
    if (a.update_here && threadIdx.x == 0) ready_seen = xwg_load64(&a.ctrl->ready);
    if (a.update_here) step_merge_clear(merge);
    block_counters_clear(counters);

    Divergence dv;
    dv.counted = false;
    dv.key = 0;
    dv.probe = OcmProbe{0, 0, false, false};
    dv.n = 0;
    bool stalled = false;
    if (b < a.B) {                                   // wave-uniform: a wave takes a sequence or none
        const DraftLane dl = load_draft_lane<false>(a, b, lane);
        const int P = a.shard_per_row[0];
        const int G = lanes_per_row(K1);
        const int grow = lane / G, gs = lane & (G - 1);
        const bool active = grow < nrows;
        const int64_t prow = (int64_t)b * K1 + (active ? grow : 0);
        StepRecord *row_rec = a.records + prow * P;
        const uint64_t rec0 = (uint64_t)prow * (uint64_t)P;
        float gm;
        int t;
        double S;
        const bool ok = acquire_row_stats_any(row_rec, rec0, P, G, gs, active, kLog2eD, a.reader_nonce, a.spin_limit, gm, t, S);
        stalled = !ok;
        if (!stalled) {
            float rmax;
            int tstar;
            double rS;
            publish_row_stats(a, b, lane, G, nrows, gm, t, S, rmax, tstar, rS);
            if (a.update_here) dv = sequence_decide<true>(a, b, lane, dl, rmax, tstar, rS, !bonus_later, counters);
            else dv = sequence_decide<false>(a, b, lane, dl, rmax, tstar, rS, !bonus_later, counters);
        } else {                                     // the records never came: say so, and report nothing as accepted
            report_stalled_sequence(a.accept_len, a.next_token, a.pos_flags, a.rej_log, b, k, lane);
            if (lane == 0) atomicAdd(&counters.v[CSD_STATUS_STALLED], 1u);
        }
        if (bonus_later && lane == 0)
            publish_word(a.seq_words + b, a.nonce, (uint64_t)b, stalled ? kSeqWordStalled : (uint64_t)(uint32_t)dv.n);
    }

    sequence_counters_and_updates(a.ctrl, ready_seen, step_ready_value(a.reader_nonce), wg == 0, (uint32_t)a.n_seq_wgs,
                                  a.update_here != 0, a.ocm, a.capacity, a.status, counters, merge, dv, verdict, a.spin_limit);
}

// Bonus-rows-last order, the workgroups at the very end of the grid: one wave per sequence takes the statistics of
// the sequence's bonus row (nothing but these outputs depends on that row) and, when the loop kept every draft
// token, the emitted token.  It waits for the bonus row's records and for the word its sequence's loop left -
// both published by workgroups earlier in the grid.  A loop that reported a stall has reported everything; a
// bonus row whose records never come is counted as a stall of its own and the emitted token, if it was to come
// from that row, reads -1.
__device__ __forceinline__ void step_bonus_rows(const EpilogueArgs &a, int wg) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int b = wg * kStepSeqWaves + (threadIdx.x >> 6);
    if (b >= a.B) return;                            // wave-uniform
    const int k = a.k, K1 = a.k + 1, P = a.shard_per_row[0];
    const int64_t row = (int64_t)b * K1 + k;
    // the word first: it has been there for a while, and its loads travel with the records' first round
    WordRecord *word = a.seq_words + b;
    uint64_t wv = 0, wc = 0;
    if (lane == 0) {
        wv = xwg_load64(&word->value);
        wc = xwg_load64(&word->check);
    }
    float gm;
    int t;
    double S;
    const bool ok = acquire_row_stats_any(a.records + row * P, (uint64_t)row * (uint64_t)P, P, kWaveSize, lane, true, kLog2eD,
                                          a.reader_nonce, a.spin_limit, gm, t, S);
    if (lane != 0) return;
    bool have_word = (wc == word_check(wv, a.reader_nonce, (uint64_t)b));
    if (have_word) xwg_store64(&word->check, 0ull);
    else have_word = acquire_word(word, a.reader_nonce, (uint64_t)b, wv, a.spin_limit);
    const bool loop_reported = have_word && wv != kSeqWordStalled;
    if (ok) {
        a.argmax[row] = t;
        if (a.row_max) a.row_max[row] = gm;
        if (a.row_sumexp) a.row_sumexp[row] = (float)S;
        if (loop_reported && (int)wv == k) a.next_token[b] = t;
    } else {
        if (loop_reported) {                         // otherwise the loop's own stall is the one that is counted
            if ((int)wv == k) a.next_token[b] = -1;
            if (a.status != nullptr) atomicAdd(&a.status[CSD_STATUS_STALLED], 1u);
        }
    }
}

template <int DT>
__global__ __launch_bounds__(kStreamWaves *kWaveSize, 4) void verify_step_kernel(StreamSource src, int V, int nsplit,
                                                                                 EpilogueArgs a) {
    __shared__ BlockCounters counters;
    __shared__ int verdict;
    __shared__ RowPartial wave_out[kStreamWaves];
    __shared__ StepMergeLds merge;
    const int g = (int)blockIdx.x;
    if (g >= a.n_stream_wgs) {                       // the streaming workgroups come first in either order
        if (g < a.n_stream_wgs + a.n_seq_wgs) step_sequences(a, g - a.n_stream_wgs, counters, merge, &verdict);
        else step_bonus_rows(a, g - a.n_stream_wgs - a.n_seq_wgs);
        return;
    }
    int row, place;                                  // this streaming workgroup's row and its place among the row's workgroups
    if (!a.order.bonus_last) {
        row = g / nsplit;
        place = g - row * nsplit;
    } else if (g < a.order.n_draft_wgs) {            // the rows of the draft positions, sequence by sequence
        const int r = g / nsplit;
        place = g - r * nsplit;
        const int b = r / a.k;
        row = b * (a.k + 1) + (r - b * a.k);
    } else {                                         // then the bonus rows
        const int g2 = g - a.order.n_draft_wgs;
        const int b = g2 / nsplit;
        place = g2 - b * nsplit;
        row = b * (a.k + 1) + a.k;
    }
    const int split = share_of_workgroup(place, row, nsplit);
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    if (a.update_here && blockIdx.x == 0 && threadIdx.x == 0) step_control_setup(a.ctrl, step_ready_value(a.nonce));
    const char *rowp = src.base0 + (int64_t)row * src.pitch0;
    const RowPartial out = stream_row_share<DT>(rowp, V, nsplit, split, wave, lane, src.scale);
    publish_workgroup_share(wave_out, out, wave, lane, a.records, (uint64_t)row * nsplit + split, a.nonce);
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
    const int64_t resident = kResidentWorkgroups;
    int tiles_per_group = 2;
    if ((int64_t)rows * ((ntr + 1) / 2) > resident) {
        for (int t = 3; t <= 4; ++t)
            if ((int64_t)rows * ((ntr + t - 1) / t) <= resident) { tiles_per_group = t; break; }
    }
    int nsplit = (p.ntiles_row + tiles_per_group - 1) / tiles_per_group;
    if (nsplit < 1) nsplit = 1;
    // A launch small enough to be resident at once even with one workgroup per tile is bound by latency, not by
    // bandwidth: every workgroup then takes ONE round of loads - a tile, or the row's remainder as a share of its
    // own (8 rows of 128256 bf16 logits, k = 5: 12.4 -> 11.4 microseconds per step).
    const bool has_rem = p.nchunks > p.ntiles_row * kTileChunks;
    const int one_round = p.ntiles_row + ((has_rem && p.ntiles_row > 0) ? 1 : 0);
    if (one_round >= 1 && (int64_t)rows * one_round <= resident) nsplit = one_round;
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
    w.words_off = (w.log_off + w.log_bytes + 255) & ~(size_t)255;
    w.words_bytes = (size_t)B * sizeof(WordRecord);
    w.total = (w.words_off + w.words_bytes + 255) & ~(size_t)255;
    return w;
}

// Which grid order a step takes.  With the bonus rows last, the sequence workgroups (which sit behind every
// streaming workgroup in either order) find the rows they need complete while the bonus rows are still being
// streamed, so the loop, the lookups and the barrier start that much earlier, and only one round trip (the bonus
// rows' records) has to follow the last streaming workgroup.  Measured per step, plain order -> bonus rows last:
// 64 sequences of 9 fp32 rows 59.2 -> 56.8 microseconds, 256 sequences of 5 bf16 rows 103.2 -> 101.9.  A launch that
// is resident all at once streams every row at the same time; the order then only adds the hand-over of the
// accepted length (one more dependent round trip when no updates are applied): such launches keep the plain order.
// (Sequence workgroups placed earlier in the grid, so that they are resident as soon as the draft positions' rows
// are complete, finish their loop well before the stream ends but take 64 places from streaming workgroups for 17
// microseconds, and their atomics land on channels that are busy streaming: measured no gain at any position.)
static std::atomic<int> g_step_order_override{0};   // test hook: 1 forces the plain order, 2 the bonus-rows-last order
void set_step_order_override(int v) { g_step_order_override.store(v, std::memory_order_relaxed); }
StepOrder make_step_order(const StreamPlan &p, int B, int k) {
    StepOrder o;
    o.n_draft_wgs = B * k * p.nsplit;
    const int force = g_step_order_override.load(std::memory_order_relaxed);
    const bool want = (force == 2) || (force == 0 && (int64_t)p.rows * p.nsplit > kResidentWorkgroups);
    o.bonus_last = (want && k >= 1 && B >= 1) ? 1 : 0;
    return o;
}

hipError_t launch_row_partials(const StreamSource &src, int dtype, int V, const StreamPlan &plan, RowPartial *partials,
                               hipStream_t stream) {
    if (plan.rows == 0) return hipSuccess;
    const dim3 grid((unsigned)(plan.rows * plan.nsplit)), block(kStreamWaves * kWaveSize);
    if (dtype == CSD_DTYPE_F32)
        hipLaunchKernelGGL(row_partials_kernel<CSD_DTYPE_F32>, grid, block, 0, stream, src, V, plan.nsplit, partials);
    else
        hipLaunchKernelGGL(row_partials_kernel<CSD_DTYPE_BF16>, grid, block, 0, stream, src, V, plan.nsplit, partials);
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
    const int n_tail_wgs = a.order.bonus_last ? a.n_seq_wgs : 0;   // the workgroups that take the bonus rows' statistics
    const dim3 grid((unsigned)(a.n_stream_wgs + a.n_seq_wgs + n_tail_wgs)), block(kStreamWaves * kWaveSize);
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
