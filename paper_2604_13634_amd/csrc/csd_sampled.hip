// Verification at a sampling temperature T > 0: Algorithm 1's loop as printed, with the uniform random
// numbers it draws handed in by the caller.
//
//   per draft position i:  p_i = softmax(target logits / T),  q_i = softmax(draft logits / T)
//     accept x~ when r <= min(1, p_i(x~)/q_i(x~))                                              (Eq. 2)
//     else draw t* from norm(max(0, p_i - q_i)) by inverting its running sum at u (ascending token id),
//          look (x~, t*) up in the memory, gate on exp(z(x~) - z(t*)) of the raw target logits (Eq. 3),
//          count the pair, then keep x~ (rescued) or stop and emit t*
//   all kept: emit a draw from p_{k+1}.
//
// Three launches on the caller's stream:
//   1. sampled_stream_kernel.  First role: the streaming pass (csd_stream.h) over the B(k+1) target rows and the
//      Bk draft rows in one grid, with the exponent scale log2(e)/T: maxima and normalisers at temperature T,
//      one record per workgroup.                                                           [HBM-bound]
//      Second role (workgroups at the end of the grid), one wave per sequence: waits for the records of its
//      rows, then p(x~), q(x~), alpha, the acceptance test; leaves for every "draw row" (a rejected position,
//      or the bonus row) the constants that turn a logit into a probability, and a list of the rows that need
//      a draw.
//   2. residual_segments_kernel, one workgroup per (row of that list, group of segments): streams the target
//      row and the draft row side by side and leaves the residual mass of every segment of 256 chunks.
//                                                                                          [HBM-bound]
//   3. sampled_tail_kernel.  First role, one wave per draw row: scans the segment masses in double, finds the
//      segment that holds u*R, re-reads that one segment, walks to the token and publishes the draw.  Second
//      role (workgroups at the end of the grid), one wave per sequence: waits for the draws of its rows, then
//      lookup, gate, accepted-prefix scan, emitted token, log, and the step's updates after a barrier of the
//      sequence workgroups (the same tail as the greedy step's single launch).
// Measured at 256 sequences, k = 4, 256000 bf16 logits, T = 1 (about 630 draw rows): 174 + 76 + 16 microseconds.
// In the last launch a draw is published 5 us after the launch began at the median and 7.4 at the latest (0.4
// row constants and segment masses, 0.6 choosing the segment, 2.6 re-reading it, 1.2 - 2 finding the token), the
// sequence waves have their draws at 8, have run the loop at 9.5, and the updates are out at 13.5.
// Positions whose acceptance test fails are all drawn (the draws do not depend on each other), although
// the loop may stop before it reaches some of them; so is the bonus token of every sequence.
#include "csd_stream.h"

namespace csd {
namespace {

constexpr int kSegLoads = 4;                          // 16-byte loads per lane and segment
constexpr int kSegChunks = kWaveSize * kSegLoads;     // chunks per segment (one wave sweeps a segment)
constexpr int kSegsPerWave = 2;                       // segments one wave takes per item: one round of loads
constexpr int kSegBlockWaves = 4;                      // waves per workgroup of the last launch
constexpr int kSegItemWaves = 4;                       // waves per workgroup of the segment kernel: one item
constexpr int kSegGrid = 1 << 22;                     // most workgroups of the segment kernel
constexpr int kNone = 0x7fffffff;

// probability of one logit from the row constants: 2^(z*scale - c) * f.  Separate roundings (no
// contraction) so that the segment pass and the locate pass see the same numbers.
__device__ __forceinline__ float prob_of(float z, float scale, float c, float f) {
    return __fmul_rn(__builtin_amdgcn_exp2f(__builtin_fmaf(z, scale, -c)), f);
}

template <int DT>
__device__ __forceinline__ u32x4 load_chunk_guarded(const char *row, int ch, int nfull, int tail) {
    using C = Chunk<DT>;
    u32x4 q = {C::kNegInfWord, C::kNegInfWord, C::kNegInfWord, C::kNegInfWord};
    if (ch < nfull) q = ((const u32x4 *)row)[ch];
    else if (ch == nfull && tail > 0) q = C::load_ragged(row, nfull * C::E, tail);
    return q;
}

// the same for the streaming pass: non-temporal, the row is not read again by this kernel
template <int DT>
__device__ __forceinline__ u32x4 stream_chunk_guarded(const char *row, int ch, int nfull, int tail) {
    using C = Chunk<DT>;
    u32x4 q = {C::kNegInfWord, C::kNegInfWord, C::kNegInfWord, C::kNegInfWord};
    if (ch < nfull) q = __builtin_nontemporal_load((const u32x4 *)row + ch);
    else if (ch == nfull && tail > 0) q = C::load_ragged(row, nfull * C::E, tail);
    return q;
}

// residual weights of one chunk: w = max(0, p - q), or p itself for the bonus row (use_q false)
template <int DT>
__device__ __forceinline__ void weights_of(const u32x4 &cp, const u32x4 &cq, bool use_q, float scale, const DrawRow &r,
                                           float (&w)[Chunk<DT>::E]) {
    using C = Chunk<DT>;
    float x[C::E];
    C::unpack(cp, x);
#pragma unroll
    for (int j = 0; j < C::E; ++j) w[j] = prob_of(x[j], scale, r.cp, r.fp);
    if (use_q) {
        float y[C::E];
        C::unpack(cq, y);
#pragma unroll
        for (int j = 0; j < C::E; ++j) w[j] = __builtin_fmaxf(__fsub_rn(w[j], prob_of(y[j], scale, r.cq, r.fq)), 0.f);
    }
}
// exclusive prefix sum over the 64 lanes, in double; `total` = the wave's sum, the same value in every lane
__device__ __forceinline__ double wave_exclusive_scan_d(double v, int lane, double &total) {
    double incl = v;
#pragma unroll
    for (int off = 1; off < kWaveSize; off <<= 1) {
        const double o = from_lane_d(incl, lane >= off ? lane - off : lane);
        if (lane >= off) incl += o;
    }
    total = from_lane_d(incl, kWaveSize - 1);
    return incl - v;
}

// ---------------------------------------------------------------------------------------------------
// Launch 1, second role: acceptance test.  One wave per sequence; lane i < k owns draft position i, lane i <= k
// draw row i.  The wave waits for the records of its 2k+1 rows (bounded; `stalled` when the wait ran out).
// Returns, per lane, whether draw row `lane` of the sequence needs a draw.
__device__ __forceinline__ bool decide_sequence(const SampledArgs &a, int b, int lane, bool &stalled) {
    const int k = a.k, K1 = a.k + 1, P = a.nsplit;
    const bool is_pos = lane < k;
    const double scale = (double)a.scale;

    int d = -1;
    bool valid = false;
    float zpd = 0.f, zqd = 0.f;
    if (is_pos) {
        d = a.draft[(int64_t)b * k + lane];
        valid = (d >= 0) && (d < a.V);
        if (valid) {
            zpd = load_logit(a.target, a.dtype, ((int64_t)b * K1 + lane) * a.target_stride + d);
            zqd = load_logit(a.draft_logits, a.dtype, ((int64_t)b * k + lane) * a.draft_stride + d);
        }
    }
    const float u_acc = is_pos ? a.u_accept[(int64_t)b * k + lane] : 0.f;
    const float u_drw = (lane < K1) ? a.u_draw[(int64_t)b * K1 + lane] : 0.f;
    int G = 1;
    while (2 * G * K1 <= kWaveSize) G *= 2;
    const int grow = lane / G, gs = lane & (G - 1);
    const int src = (lane < K1 ? lane : 0) * G;          // lane i takes the statistics of row i

    float gm;
    int gt;
    double gS;
    const int64_t prow = (int64_t)b * K1 + (grow < K1 ? grow : 0);
    bool ok = acquire_row_stats_any(a.records + prow * P, (uint64_t)prow * (uint64_t)P, P, G, gs, grow < K1, scale, a.reader_nonce,
                                    a.spin_limit, gm, gt, gS);
    const float mp = from_lane_f(gm, src);
    const int tp = from_lane_i(gt, src);
    const double Sp = from_lane_d(gS, src);
    float mq = 0.f;
    double Sq = 1.0;
    if (k > 0) {
        const int64_t qrow = (int64_t)a.B * K1 + (int64_t)b * k + (grow < k ? grow : 0);   // draft rows follow the target rows
        ok = acquire_row_stats_any(a.records + qrow * P, (uint64_t)qrow * (uint64_t)P, P, G, gs, grow < k, scale, a.reader_nonce,
                                   a.spin_limit, gm, gt, gS) && ok;
        mq = from_lane_f(gm, src);
        Sq = from_lane_d(gS, src);
    }
    stalled = !ok;
    if (stalled) return false;

    bool rejected = false;
    if (is_pos) {
        double pd = 0.0, qd = 0.0, alpha = 0.0;
        rejected = true;                                   // an id outside the vocabulary never passes
        if (valid) {
            pd = exp2(((double)zpd - (double)mp) * scale) / Sp;
            qd = exp2(((double)zqd - (double)mq) * scale) / Sq;
            alpha = (qd <= 0.0) ? 1.0 : fmin(1.0, pd / qd);
            rejected = (double)u_acc > alpha;
        }
        const int64_t o = (int64_t)b * k + lane;
        if (a.alpha) a.alpha[o] = (float)alpha;
        if (a.p_draft) a.p_draft[o] = (float)pd;
        if (a.q_draft) a.q_draft[o] = (float)qd;
        a.pos_zpd[o] = zpd;
        a.pos_state[o] = (uint8_t)((rejected ? 1 : 0) | (valid ? 2 : 0));
    }
    if (lane < K1) {
        DrawRow r;
        r.need = (lane == k) ? 1 : ((rejected && valid) ? 1 : 0);
        r.fallback = tp;
        r.cp = mp * a.scale;                               // float reference exponent near m*scale ...
        r.fp = (float)(exp2((double)r.cp - (double)mp * scale) / Sp);   // ... and what it leaves out, with 1/S
        r.cq = 0.f;
        r.fq = 0.f;
        if (lane < k) {
            r.cq = mq * a.scale;
            r.fq = (float)(exp2((double)r.cq - (double)mq * scale) / Sq);
        }
        r.u = u_drw;
        r.pad = 0.f;
        a.rows[(int64_t)b * K1 + lane] = r;
        return r.need != 0;
    }
    return false;
}

// nothing of this sequence is drawn, and the last launch's sequence wave reports it as stalled
__device__ __forceinline__ void mark_sequence_stalled(const SampledArgs &a, int b, int lane) {
    const int K1 = a.k + 1;
    if (lane < K1) {
        DrawRow r = {(lane == a.k) ? 2 : 0, 0, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        a.rows[(int64_t)b * K1 + lane] = r;
    }
}

// Launch 1: workgroups [0, n_stream_wgs) stream the 2k+1 rows of every sequence (target rows first, then draft
// rows) and leave one record each; the workgroups after them take four sequences each, wait for their rows'
// records and run the acceptance test, as the greedy step's single launch does with its sequence logic.  The rows
// that need a draw go on a list (order immaterial), so that the second streaming pass has work for them only:
// one LDS add per wave, one global add per workgroup.  The list's length is zeroed by the first workgroup of the
// launch, which then says so in the list's control head; a workgroup adds to it only after seeing that.
template <int DT>
__global__ __launch_bounds__(kStreamWaves *kWaveSize, 4) void sampled_stream_kernel(StreamSource src, int V, SampledArgs a) {
    __shared__ RowPartial wave_out[kStreamWaves];
    __shared__ unsigned int blk_count, blk_base;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    if ((int)blockIdx.x < a.n_stream_wgs) {
        const int row = blockIdx.x / a.nsplit;
        const int split = share_of_workgroup((int)blockIdx.x - row * a.nsplit, row, a.nsplit);
        if (blockIdx.x == 0 && threadIdx.x == 0) step_control_setup(a.list_ctrl, step_ready_value(a.nonce));
        const char *rowp = (row < src.rows0) ? src.base0 + (int64_t)row * src.pitch0
                                             : src.base1 + (int64_t)(row - src.rows0) * src.pitch1;
        const RowPartial out = stream_row_share<DT>(rowp, V, a.nsplit, split, wave, lane, src.scale);
        publish_workgroup_share(wave_out, out, wave, lane, a.records, (uint64_t)row * a.nsplit + split, a.nonce);
        return;
    }
    const int b = ((int)blockIdx.x - a.n_stream_wgs) * kStreamWaves + wave;
    uint64_t ready_seen = 0;
    if (threadIdx.x == 0) {
        ready_seen = xwg_load64(&a.list_ctrl->ready);    // asked for early, looked at late
        blk_count = 0;
        blk_base = kNone;
    }
    __syncthreads();
    bool need = false, stalled = false;
    if (b < a.B) need = decide_sequence(a, b, lane, stalled);      // wave-uniform: a wave takes a sequence or none
    const uint64_t mask = __builtin_amdgcn_ballot_w64(need);
    unsigned int off = 0;
    if (lane == 0 && mask) off = atomicAdd(&blk_count, (unsigned int)__builtin_popcountll(mask));
    off = __builtin_amdgcn_readfirstlane(off);
    __syncthreads();
    if (threadIdx.x == 0 && blk_count) {
        const uint64_t ready_value = step_ready_value(a.reader_nonce);
        bool good = true;
        for (uint32_t spin = 0; ready_seen != ready_value; ++spin) {
            if (spin >= a.spin_limit) { good = false; break; }
            __builtin_amdgcn_s_sleep(kSpinSleep);
            ready_seen = xwg_load64(&a.list_ctrl->ready);
        }
        if (good) blk_base = __hip_atomic_fetch_add(&a.list_ctrl->arrivals, blk_count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    const bool listed = blk_base != (unsigned int)kNone;
    if (need && listed)
        a.work_rows[blk_base + off + (unsigned int)__builtin_popcountll(mask & ((1ull << lane) - 1ull))] = b * (a.k + 1) + lane;
    if (b < a.B && (stalled || (mask && !listed))) {     // wave-uniform
        mark_sequence_stalled(a, b, lane);
        if (lane == 0 && a.status != nullptr) atomicAdd(&a.status[CSD_STATUS_STALLED], 1u);
    }
}

// ---------------------------------------------------------------------------------------------------
// Launch 2: residual mass per segment, for the rows on the list only.  One workgroup per item (row of the list,
// group of segments); the grid is sized for every row needing a draw (up to kSegGrid workgroups, which then take
// several items each) and the workgroups beyond the list's end leave at once.  (A fixed grid of 4096 workgroups
// walking the items measured 1.5 % slower on the whole step, workgroups of 1, 2 and 8 waves 1 - 2.5 % slower than
// these 4.)
template <int DT>
__global__ __launch_bounds__(kSegItemWaves *kWaveSize) void residual_segments_kernel(SampledArgs a) {
    using C = Chunk<DT>;
    const int groups = (a.nseg + kSegItemWaves * kSegsPerWave - 1) / (kSegItemWaves * kSegsPerWave);
    const unsigned int items = a.list_ctrl->arrivals * (unsigned int)groups;
    if (blockIdx.x == 0 && threadIdx.x == 0) xwg_store64(&a.list_ctrl->ready, 0ull);   // a replay of this step waits for its own
    for (unsigned int item = blockIdx.x; item < items; item += gridDim.x) {   // one turn, but for grids beyond kSegGrid
        const int j = a.work_rows[item / groups];
        // rotated by the list position for the reason share_of_workgroup gives: the last group of a row is the short one
        const int group = share_of_workgroup((int)(item % groups), (int)(item / groups), groups);
        const DrawRow r = a.rows[j];
        const int lane = threadIdx.x & (kWaveSize - 1);
        const int wave = threadIdx.x >> 6;
        const int K1 = a.k + 1;
        const int b = j / K1, i = j - b * K1;
        const bool use_q = i < a.k;
        const int esz = (DT == CSD_DTYPE_F32) ? 4 : 2;
        const char *prow = (const char *)a.target + (int64_t)j * a.target_stride * esz;
        const char *qrow = use_q ? (const char *)a.draft_logits + ((int64_t)b * a.k + i) * a.draft_stride * esz : prow;
        const int nfull = a.V / C::E, tail = a.V - nfull * C::E;
        const int seg0 = (group * kSegItemWaves + wave) * kSegsPerWave;
        // two segments at a time: all their loads (2 x kSegLoads per tensor) are issued before any arithmetic
        for (int s = seg0; s < seg0 + kSegsPerWave && s < a.nseg; s += 2) {
            constexpr int N = 2 * kSegLoads;
            u32x4 qp[N], qq[N];
            if ((s + 2) * kSegChunks <= nfull) {                            // both segments are whole chunks of the row: no guards
#pragma unroll
                for (int u = 0; u < N; ++u) {
                    const int ch = s * kSegChunks + u * kWaveSize + lane;   // segment s+1 follows segment s in memory
                    qp[u] = __builtin_nontemporal_load((const u32x4 *)prow + ch);
                    if (use_q) qq[u] = __builtin_nontemporal_load((const u32x4 *)qrow + ch);
                }
            } else {
#pragma unroll
                for (int u = 0; u < N; ++u) {
                    const int ch = s * kSegChunks + u * kWaveSize + lane;
                    qp[u] = stream_chunk_guarded<DT>(prow, ch, nfull, tail);
                    if (use_q) qq[u] = stream_chunk_guarded<DT>(qrow, ch, nfull, tail);
                }
            }
            float sum[2] = {0.f, 0.f};
#pragma unroll
            for (int u = 0; u < N; ++u) {
                float w[C::E];
                weights_of<DT>(qp[u], qq[u], use_q, a.scale, r, w);
#pragma unroll
                for (int e = 0; e < C::E; ++e) sum[u / kSegLoads] += w[e];
            }
            const float s0 = wave_allreduce_f(sum[0], AddF()), s1 = wave_allreduce_f(sum[1], AddF());
            if (lane == 0) {
                a.segsum[(int64_t)j * a.nseg + s] = s0;
                if (s + 1 < a.nseg) a.segsum[(int64_t)j * a.nseg + s + 1] = s1;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Launch 3, first role: invert the running sum.  One wave per draw row j; returns the drawn token (-1 when the
// row needs no draw) in every lane and writes it to the tstar / bonus output.
template <int DT>
__device__ __forceinline__ int locate_draw(const SampledArgs &a, int64_t j, int lane) {
    using C = Chunk<DT>;
    const int K1 = a.k + 1;
    const int b = (int)(j / K1), i = (int)(j - (int64_t)b * K1);
    int32_t *out = (i < a.k) ? &a.tstar[(int64_t)b * a.k + i] : &a.bonus[b];
    // ---- which segment: lane l owns segments [l*per, (l+1)*per).  Up to four per lane (every vocabulary below
    // half a million bf16 logits) are fetched together with the row's constants, before it is known whether the
    // row needs a draw at all: one memory round trip, not two, and no second read of them below.
    const float *seg = a.segsum + j * a.nseg;
    const int per = (a.nseg + kWaveSize - 1) / kWaveSize;
    const int s0 = lane * per;
    constexpr int kSegRegs = 4;
    float sv[kSegRegs];
#pragma unroll
    for (int u = 0; u < kSegRegs; ++u) sv[u] = (per <= kSegRegs && u < per && s0 + u < a.nseg) ? seg[s0 + u] : 0.f;
    const DrawRow r = a.rows[j];
    if (r.need != 1) {
        if (lane == 0) *out = -1;
        return -1;
    }
    double local = 0.0;
    if (per <= kSegRegs) {
#pragma unroll
        for (int u = 0; u < kSegRegs; ++u) local += (double)sv[u];          // absent ones are zero
    } else {
        for (int s = s0; s < s0 + per && s < a.nseg; ++s) local += (double)seg[s];
    }
    double R;
    const double before = wave_exclusive_scan_d(local, lane, R);
    int result = -1;
    if (R > 0.0) {
        const double target = (double)r.u * R;
        int found = kNone, lastpos = -1;
        double base = 0.0, acc = before;
        auto visit = [&](int s, double v) {
            if (v > 0.0) lastpos = s;
            if (found == kNone && v > 0.0 && acc + v > target) {    // a segment without mass is never chosen
                found = s;
                base = acc;
            }
            acc += v;
        };
        if (per <= kSegRegs) {
#pragma unroll
            for (int u = 0; u < kSegRegs; ++u) visit(s0 + u, (double)sv[u]);
        } else {
            for (int s = s0; s < s0 + per && s < a.nseg; ++s) visit(s, (double)seg[s]);
        }
        int sstar = wave_allreduce_i(found, MinI());
        if (sstar == kNone) {                              // rounding at the very end of the row: last segment with mass
            sstar = -wave_allreduce_i(-lastpos, MinI());
            base = 0.0;
            found = kNone - 1;                             // nobody owns `base`: walk the segment from its start with rem = +inf
        }
        const int owner = sstar / per;
        // `base` comes from the owner's serial adds, `target` was compared against a tree scan: clamp what is
        // left at zero so that the walk below starts inside the segment
        double rem = (found == kNone - 1) ? INFINITY : fmax(target - from_lane_d(base, owner), 0.0);
        // ---- inside the segment, in token order: load u, then lane, then element
        const int esz = (DT == CSD_DTYPE_F32) ? 4 : 2;
        const bool use_q = i < a.k;
        const char *prow = (const char *)a.target + j * a.target_stride * esz;
        const char *qrow = use_q ? (const char *)a.draft_logits + ((int64_t)b * a.k + i) * a.draft_stride * esz : prow;
        const int nfull = a.V / C::E, tail = a.V - nfull * C::E;
        int last_tok = -1;
        u32x4 cp[kSegLoads], cq[kSegLoads];                // the whole segment's loads first: one latency, not four
#pragma unroll
        for (int u = 0; u < kSegLoads; ++u) {
            const int ch = sstar * kSegChunks + u * kWaveSize + lane;
            cp[u] = load_chunk_guarded<DT>(prow, ch, nfull, tail);
            cq[u] = use_q ? load_chunk_guarded<DT>(qrow, ch, nfull, tail) : cp[u];
        }
        // the four running sums (one per load) are independent: taken together, their shuffles overlap
        float w[kSegLoads][C::E];
        double lsum[kSegLoads], excl[kSegLoads], tot[kSegLoads];
        int my_last[kSegLoads];
#pragma unroll
        for (int u = 0; u < kSegLoads; ++u) {
            const int ch = sstar * kSegChunks + u * kWaveSize + lane;
            weights_of<DT>(cp[u], cq[u], use_q, a.scale, r, w[u]);
            lsum[u] = 0.0;
            my_last[u] = -1;
#pragma unroll
            for (int e = 0; e < C::E; ++e) {
                lsum[u] += (double)w[u][e];
                if (w[u][e] > 0.f) my_last[u] = ch * C::E + e;
            }
            last_tok = my_last[u] > last_tok ? my_last[u] : last_tok;
        }
#pragma unroll
        for (int u = 0; u < kSegLoads; ++u) excl[u] = wave_exclusive_scan_d(lsum[u], lane, tot[u]);
#pragma unroll
        for (int u = 0; u < kSegLoads; ++u) {
            if (result >= 0) break;
            const int ch = sstar * kSegChunks + u * kWaveSize + lane;
            const uint64_t hit = __builtin_amdgcn_ballot_w64(lsum[u] > 0.0 && excl[u] + lsum[u] > rem);   // only lanes holding mass
            if (hit) {
                const int L = (int)__builtin_ctzll(hit);
                int tok = my_last[u];
                if (lane == L) {
                    double c = excl[u];
                    bool done = false;
#pragma unroll
                    for (int e = 0; e < C::E; ++e) {
                        c += (double)w[u][e];
                        if (!done && w[u][e] > 0.f && c > rem) {   // never a token outside the residual's support
                            tok = ch * C::E + e;
                            done = true;
                        }
                    }
                }
                result = from_lane_i(tok, L);
            } else {
                rem -= tot[u];
            }
        }
        if (result < 0) result = -wave_allreduce_i(-last_tok, MinI());   // rounding: the segment's last token with mass
    }
    if (result < 0) result = r.fallback;                   // no residual mass at all: the target's own choice
    if (lane == 0) *out = result;
    return result;
}

// ---------------------------------------------------------------------------------------------------
// Launch 3, second role: the loop itself.  One wave per sequence; it waits for the draws of its k+1 rows, which
// the first role's waves of the same launch publish.
__device__ __forceinline__ Divergence sampled_sequence(const SampledArgs &a, int b, int lane, BlockCounters &counters, bool &stalled,
                                                       bool &stalled_before) {
    const int k = a.k, K1 = a.k + 1;
    const bool is_pos = lane < k;
    int d = -1;
    bool valid = false, rejected = false;
    float zpd = 0.f, zpt = 0.f;
    if (is_pos) {                                          // from the acceptance test's launch: there before this one began
        const int64_t o = (int64_t)b * k + lane;
        d = a.draft[o];
        const uint8_t st = a.pos_state[o];
        rejected = st & 1;
        valid = st & 2;
        zpd = a.pos_zpd[o];
    }
    const DrawRow *mine_row = &a.rows[(int64_t)b * K1 + (lane < K1 ? lane : 0)];
    const int fallback = mine_row->fallback;
    stalled_before = from_lane_i(mine_row->need, k) == 2;     // the first launch gave this sequence up (and counted it)
    Divergence out;
    out.counted = false;
    out.key = 0;
    out.probe = OcmProbe{0, 0, false, false};
    out.n = 0;
    stalled = stalled_before;
    if (stalled_before) return out;
    // the draws of this sequence's rows: lane i takes row i's
    int t = -1;
    bool got = true;
    if (lane < K1) {
        uint64_t v = 0;
        const uint64_t rec = (uint64_t)b * K1 + lane;
        got = acquire_word(a.draws + rec, a.reader_nonce, rec, v, a.spin_limit);
        t = (int)(uint32_t)v;
    }
    stalled = __builtin_amdgcn_ballot_w64(!got) != 0ull;
    if (stalled) return out;
    const int bonus = from_lane_i(t, k);
    if (is_pos && rejected && valid) zpt = load_logit(a.target, a.dtype, ((int64_t)b * K1 + lane) * a.target_stride + t);

    const bool diverges = is_pos && rejected && valid;
    // Eq. 3 on the raw target logits
    const double ratio = diverges ? exp2(((double)zpd - (double)zpt) * 1.4426950408889634) : 0.0;
    if (is_pos && a.ratio) a.ratio[(int64_t)b * k + lane] = (float)ratio;
    out.key = CSD_OCM_KEY((uint32_t)(diverges ? d : 0), (uint32_t)(diverges ? t : 0));
    bool is_freq = false;
    if (diverges && a.ocm != nullptr) {
        if (a.update_here) {
            out.probe = ocm_probe(a.ocm, a.capacity, out.key);
            is_freq = out.probe.count >= a.lambda;
        } else {
            is_freq = (a.lambda == 0) ? true : (ocm_lookup(a.ocm, a.capacity, out.key) >= a.lambda);
        }
    }
    const bool is_safe = diverges && (ratio >= (double)a.tau);
    const bool ok = is_pos && (!rejected || (is_freq && is_safe));

    const uint64_t fail = __builtin_amdgcn_ballot_w64(is_pos && !ok) | (1ull << k);
    const int n = (int)__builtin_ctzll(fail);
    const bool processed = is_pos && (lane <= n);
    const bool counted = processed && diverges;
    out.counted = counted;
    // emitted token: the stopping position's t* (the target argmax when its draft id was invalid), else the bonus draw
    int mine = diverges ? t : fallback;
    if (lane == k) mine = bonus;
    const int next = from_lane_i(mine, n);

    if (is_pos) {
        const int64_t o = (int64_t)b * k + lane;
        if (a.pos_flags) {
            uint8_t f = 0;
            if (processed) {
                if (!rejected) f = CSD_POS_MATCH | CSD_POS_ACCEPTED;
                else if (diverges)
                    f = CSD_POS_COUNTED | (is_freq ? CSD_POS_FREQ : 0) | (is_safe ? CSD_POS_SAFE : 0) |
                        (ok ? CSD_POS_ACCEPTED : 0);
            }
            a.pos_flags[o] = f;
        }
        if (a.rej_log) xwg_store64(&a.rej_log[o], counted ? out.key : CSD_OCM_EMPTY);
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

// Launch 3: workgroups [0, n_loc_wgs) invert the running sums (one wave per draw row) and publish each draw; the
// workgroups after them take four sequences each, wait for their rows' draws and run the loop, then apply the
// updates as the greedy step does (sequence_counters_and_updates).  Workgroups of a launch start in index order,
// so a sequence wave only waits for waves that have been started.
template <int DT>
__global__ __launch_bounds__(kSegBlockWaves *kWaveSize) void sampled_tail_kernel(SampledArgs a) {
    __shared__ BlockCounters counters;
    __shared__ StepMergeLds merge;
    __shared__ int verdict;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int K1 = a.k + 1;
    if ((int)blockIdx.x < a.n_loc_wgs) {
        if (a.update_here && blockIdx.x == 0 && threadIdx.x == 0) step_control_setup(a.ctrl, step_ready_value(a.nonce));
        const int64_t j = (int64_t)blockIdx.x * kSegBlockWaves + wave;
        if (j >= (int64_t)a.B * K1) return;
        const int result = locate_draw<DT>(a, j, lane);
        if (lane == 0) publish_word(a.draws + j, a.nonce, (uint64_t)j, (uint64_t)(uint32_t)result);
        return;
    }
    const int wg = (int)blockIdx.x - a.n_loc_wgs;
    const int n_seq_wgs = (int)gridDim.x - a.n_loc_wgs;
    const int b = wg * kSegBlockWaves + wave;
    uint64_t ready_seen = 0;
    if (a.update_here && threadIdx.x == 0) ready_seen = xwg_load64(&a.ctrl->ready);
    if (a.update_here) step_merge_clear(merge);
    block_counters_clear(counters);
    Divergence dv;
    dv.counted = false;
    dv.key = 0;
    dv.probe = OcmProbe{0, 0, false, false};
    dv.n = 0;
    if (b < a.B) {                                         // wave-uniform: a wave takes a sequence or none
        bool stalled = false, stalled_before = false;
        dv = sampled_sequence(a, b, lane, counters, stalled, stalled_before);
        if (stalled) {                                     // the draws never came: say so, and report nothing as accepted
            report_stalled_sequence(a.accept_len, a.next_token, a.pos_flags, a.rej_log, b, a.k, lane);
            if (lane == 0 && !stalled_before) atomicAdd(&counters.v[CSD_STATUS_STALLED], 1u);
        }
    }
    sequence_counters_and_updates(a.ctrl, ready_seen, step_ready_value(a.reader_nonce), wg == 0, (uint32_t)n_seq_wgs,
                                  a.update_here != 0, a.ocm, a.capacity, a.status, counters, merge, dv, &verdict, a.spin_limit);
}

}  // namespace

int sampled_segments(int V, int dtype) {
    const int e = (dtype == CSD_DTYPE_F32) ? 4 : 8;
    const int nchunks = (V + e - 1) / e;
    return (nchunks + kSegChunks - 1) / kSegChunks;
}

hipError_t launch_sampled_step(const StreamSource &src, const SampledArgs &a, hipStream_t stream) {
    if (a.B == 0) return hipSuccess;
    const int K1 = a.k + 1;
    const dim3 first_grid((unsigned)(a.n_stream_wgs + (a.B + kStreamWaves - 1) / kStreamWaves)), first_block(kStreamWaves * kWaveSize);
    const int per_block = kSegItemWaves * kSegsPerWave;
    const int64_t max_items = (int64_t)a.B * K1 * ((a.nseg + per_block - 1) / per_block);
    const dim3 seg_grid((unsigned)(max_items < kSegGrid ? max_items : kSegGrid));
    const dim3 tail_grid((unsigned)(a.n_loc_wgs + (a.B + kSegBlockWaves - 1) / kSegBlockWaves)), tail_block(kSegBlockWaves * kWaveSize);
    hipError_t e;
    if (a.dtype == CSD_DTYPE_F32) {
        hipLaunchKernelGGL(sampled_stream_kernel<CSD_DTYPE_F32>, first_grid, first_block, 0, stream, src, a.V, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(residual_segments_kernel<CSD_DTYPE_F32>, seg_grid, dim3(kSegItemWaves * kWaveSize), 0, stream, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(sampled_tail_kernel<CSD_DTYPE_F32>, tail_grid, tail_block, 0, stream, a);
    } else {
        hipLaunchKernelGGL(sampled_stream_kernel<CSD_DTYPE_BF16>, first_grid, first_block, 0, stream, src, a.V, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(residual_segments_kernel<CSD_DTYPE_BF16>, seg_grid, dim3(kSegItemWaves * kWaveSize), 0, stream, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(sampled_tail_kernel<CSD_DTYPE_BF16>, tail_grid, tail_block, 0, stream, a);
    }
    return hipGetLastError();
}

int sampled_locate_workgroups(int B, int k) { return (int)(((int64_t)B * (k + 1) + kSegBlockWaves - 1) / kSegBlockWaves); }
int sampled_sequence_workgroups(int B) { return (B + kSegBlockWaves - 1) / kSegBlockWaves; }

}  // namespace csd
