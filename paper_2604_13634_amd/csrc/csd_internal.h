// Internal declarations shared by the kernels and the C ABI (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "csd.h"

namespace csd {

// One wave's result for its share of a logits row (public layout, see csd.h).
using RowPartial = csd_row_partial;
static_assert(sizeof(RowPartial) == 16, "partials are read and written as 16-byte records");

constexpr int kWaveSize = 64;
constexpr int kStreamWaves = 4;              // waves per workgroup of the verify kernel
constexpr int kStreamUnroll = 8;             // 16-byte loads in flight per lane
constexpr int kTileChunks = kStreamWaves * kWaveSize * kStreamUnroll;   // 16-byte chunks per workgroup iteration (32 KiB)

// Launch plan of the streaming pass; a pure function of the shape so that the workspace size query and
// the launch agree.  A row's whole tiles are cut into `nsplit` contiguous runs, one per workgroup; the last
// workgroup also takes the remainder (chunks past the last whole tile, ragged one included).
struct StreamPlan {
    int rows;              // verify rows, B * (k + 1)
    int elems_per_chunk;   // 4 (fp32) or 8 (bf16) logits per 16-byte chunk
    int nchunks;           // chunks per row, the ragged last one included
    int ntiles_row;        // whole tiles of whole chunks per row
    int nsplit;            // workgroups per row
    int partials_per_row;  // nsplit * kStreamWaves: one partial per wave
};

StreamPlan make_stream_plan(int rows, int V, int dtype);

// What a streaming workgroup of the single-launch step hands to the sequence waves of the same launch: the row
// partial of its four waves together (w0 = m | cref << 32, w1 = s | idx << 32) and a check word, a 64-bit hash of the two data words, of a
// per-call number and of the record's index.  A reader takes a record as written once the check holds (a torn
// read fails it); arbitrary memory passes with probability 2^-64, so the workspace needs no initialisation.
// Readers zero the check word after use: a replay of the same call (a captured graph carries the same per-call
// number) then starts from records that do not pass.
struct StepRecord {
    uint64_t w0, w1, check, pad;
};
static_assert(sizeof(StepRecord) == 32, "records are 32 bytes");

// A published word: a 64-bit value with a check word beside it (a hash of the value, of a per-call number and of
// the record's index).  What the draw waves of the sampled step's last launch hand to its sequence waves.
struct WordRecord {
    uint64_t value, check;
};

// Head of the csd_verify workspace.  `arrivals` is the counter behind the barrier of the sequence workgroups;
// the first workgroup of every launch that uses the barrier zeroes it and then writes a word derived from the
// call's number into `ready`; the sequence workgroups count themselves in once they see that word, and clear
// it after the barrier.  The head may hold anything before a call.
struct StepControl {
    uint64_t ready;
    uint32_t arrivals;
    uint32_t pad;
};

// csd_verify workspace: [control | records | rejection log | sequence words].  Nothing in it outlives a call.
struct WorkspaceLayout {
    size_t ticket_off;                       // the control head (the ticket of the two-launch forms lives here too)
    size_t partials_off, partials_bytes;     // StepRecord per streaming workgroup
    size_t log_off, log_bytes;
    size_t words_off, words_bytes;           // WordRecord per sequence (bonus-rows-last order only)
    size_t total;
};

WorkspaceLayout make_workspace_layout(const StreamPlan &p, int B, int k);

// Grid order of the single-launch step.  Plain order: every row's streaming workgroups in row order, then the
// sequence workgroups.  Bonus-rows-last order (launches too large to be resident at once): the streaming workgroups
// of the draft positions' rows, those of the bonus rows, the sequence workgroups (which take the draft positions'
// rows only), and one more set of workgroups that takes the bonus rows' statistics.  A pure function of the shape.
struct StepOrder {
    int bonus_last;        // 0: plain order
    int n_draft_wgs;       // streaming workgroups of the draft positions' rows (B * k * nsplit)
};
StepOrder make_step_order(const StreamPlan &p, int B, int k);
void set_step_order_override(int v);                 // test hook: 0 by shape, 1 always plain, 2 bonus rows last whenever k >= 1
constexpr int kResidentWorkgroups = 4 * 256;         // streaming workgroups resident at once (four per compute unit)

// Everything the per-sequence epilogue and the update phase need.
struct EpilogueArgs {
    const void *logits;
    int dtype;
    int64_t row_stride;      // elements
    const int32_t *draft;
    int B, k, V;
    float tau;
    uint32_t lambda;
    uint64_t *ocm;           // NULL: no memory
    uint64_t capacity;
    // row partials: n_shards vocabulary shards (1 for csd_verify), shard s covering token ids from shard_base[s]
    int sharded;               // 1: csd_verify_shards (several partial sets, draft logits from draft_logit)
    int n_shards;
    const RowPartial *shard_partials[CSD_MAX_SHARDS];
    int shard_per_row[CSD_MAX_SHARDS];
    int shard_base[CSD_MAX_SHARDS];
    const float *draft_logit;  // [B][k] logit of each draft token when the logits are not at hand (shards), else NULL
    int32_t *accept_len;
    int32_t *next_token;
    int32_t *argmax;
    float *row_max;
    float *row_sumexp;
    float *ratio;
    float *p_draft;
    uint8_t *pos_flags;
    uint64_t *rej_log;       // user log or workspace log; NULL when nothing needs it
    uint32_t *status;
    uint32_t *batch_ticket;  // [2]: the ticket, and a spare counter; zero when the finish kernel starts
    int apply_updates;
    // single-launch step only
    StepRecord *records;     // [rows][nsplit]: one per streaming workgroup
    StepControl *ctrl;
    uint64_t nonce;          // per-call number behind the records' check words
    uint64_t reader_nonce;   // the same number as the readers use it (a test hook can make them differ: nothing then passes)
    uint32_t spin_limit;     // polls after which a wait inside the launch gives up
    int n_stream_wgs;        // streaming workgroups of the launch (plain order: workgroups [0, n_stream_wgs); the rest take sequences)
    int update_here;         // 1: the sequence waves apply their own increments after a barrier among their workgroups
    int n_seq_wgs;           // sequence workgroups
    StepOrder order;         // where they sit in the grid
    WordRecord *seq_words;   // [B] bonus-rows-last order: what a sequence's loop hands to the wave that takes its bonus row
};

// Where the rows of a streaming launch live: rows [0, rows0) in tensor 0, the others in tensor 1
// (pitches in bytes), and the exponent scale log2(e) / temperature the sums are made with.
struct StreamSource {
    const char *base0;
    int64_t pitch0;
    int rows0;
    const char *base1;
    int64_t pitch1;
    float scale;
};

// ---- verification at a sampling temperature (csd_sampled.hip)
// What the residual kernels need for one draw row (a rejected draft position, or the bonus row).
struct DrawRow {
    int32_t need;      // 0: nothing is drawn for this row; 1: a draw; 2 (on a sequence's bonus row only): the
                       // sequence's first-launch wait ran out, nothing of it is drawn and its loop is not run
    int32_t fallback;  // the target row's argmax: reported when the residual has no mass, or the draft id was invalid
    float cp, fp;      // p_v = 2^(z_v * scale - cp) * fp
    float cq, fq;      // q_v likewise; unused for the bonus row, which draws from p itself
    float u;           // the uniform of this draw
    float pad;
};
static_assert(sizeof(DrawRow) == 32, "draw rows are 32-byte records");

struct SampledArgs {
    const void *target;        // [B][k+1][V]
    const void *draft_logits;  // [B][k][V]
    int dtype;
    int64_t target_stride, draft_stride;   // elements
    const int32_t *draft;
    int B, k, V;
    float scale;               // log2(e) / temperature, as the streaming pass used it
    const float *u_accept;     // [B][k]
    const float *u_draw;       // [B][k+1]
    float tau;
    uint32_t lambda;
    uint64_t *ocm;
    uint64_t capacity;
    StepRecord *records;       // one per streaming workgroup of the first launch: target rows first, then draft rows
    int nsplit;                // streaming workgroups (records) per row
    int n_stream_wgs;          // streaming workgroups of the first launch; its acceptance-test workgroups follow
    int nseg;                  // segments per row
    DrawRow *rows;             // [B][k+1]
    StepControl *list_ctrl;    // `arrivals` is the number of rows that need a draw; zeroed and announced by the
                               // first launch's first workgroup, the announcement cleared by the second launch
    int32_t *work_rows;        // [B][k+1] their indices, in no particular order
    float *segsum;             // [B][k+1][nseg]
    float *pos_zpd;            // [B][k] target logit of the draft token
    uint8_t *pos_state;        // [B][k] bit0 acceptance test failed, bit1 draft id valid
    int32_t *tstar;            // [B][k] user buffer or workspace
    int32_t *bonus;            // [B]    user buffer or workspace
    int32_t *accept_len;
    int32_t *next_token;
    float *alpha;
    float *p_draft;
    float *q_draft;
    float *ratio;
    uint8_t *pos_flags;
    uint64_t *rej_log;
    uint32_t *status;
    WordRecord *draws;         // [B][k+1] the draws, published inside the last launch
    StepControl *ctrl;         // barrier state of the last launch's sequence workgroups
    uint64_t nonce;            // per-call number behind the draws' check words
    uint64_t reader_nonce;     // the same number as the readers use it (a test hook can make them differ)
    uint32_t spin_limit;       // polls after which a wait inside the launch gives up
    int n_loc_wgs;             // workgroups of the last launch that invert running sums; the sequence workgroups follow
    int update_here;           // 1: the sequence waves apply their own increments after a barrier among their workgroups
};

struct SampledWorkspace {
    size_t ticket_off, partials_off, rows_off, work_off, segsum_off, zpd_off, state_off, tstar_off, bonus_off, draws_off, log_off,
        total;
};
int sampled_locate_workgroups(int B, int k);
int sampled_sequence_workgroups(int B);
int sampled_segments(int V, int dtype);
hipError_t launch_sampled_step(const StreamSource &src, const SampledArgs &a, hipStream_t stream);

// kernel launchers (enqueue only; return hipGetLastError())
hipError_t launch_row_partials(const StreamSource &src, int dtype, int V, const StreamPlan &plan, RowPartial *partials,
                               hipStream_t stream);
hipError_t launch_finish(const EpilogueArgs &a, hipStream_t stream);
hipError_t launch_verify_step(const StreamSource &src, int dtype, int V, const StreamPlan &plan, const EpilogueArgs &a,
                              hipStream_t stream);
constexpr int kStepSeqWaves = kStreamWaves;      // sequences per workgroup of the single-launch step's second role
constexpr int kMaxBarrierWorkgroups = 64;        // sequence workgroups that may wait for each other inside a launch
hipError_t launch_zero_ticket(uint32_t *ticket, hipStream_t stream);
hipError_t launch_shard_draft_logits(const void *logits, int dtype, int64_t row_stride, int B, int k, int V_shard, int base,
                                     const int32_t *draft, float *draft_logit, hipStream_t stream);
hipError_t launch_ocm_update(uint64_t *ocm, uint64_t capacity, const uint64_t *keys, const uint32_t *weights, uint64_t n,
                             const uint64_t *n_dev, uint32_t *status, hipStream_t stream);
hipError_t launch_ocm_reset(uint64_t *ocm, uint64_t capacity, hipStream_t stream);
hipError_t launch_ocm_merge(uint64_t *dst, uint64_t dst_capacity, const uint64_t *src, uint64_t src_capacity,
                            uint32_t *status, hipStream_t stream);
hipError_t launch_ocm_export(const uint64_t *ocm, uint64_t capacity, uint64_t *keys_out, uint32_t *counts_out,
                             uint64_t max_entries, uint64_t *n_out, hipStream_t stream);
hipError_t launch_ocm_lookup(const uint64_t *ocm, uint64_t capacity, const uint64_t *keys, uint32_t *counts, uint64_t n,
                             hipStream_t stream);

}  // namespace csd
