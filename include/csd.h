/*
 * csd.h - C ABI of the batched verification step of Calibrated Speculative Decoding (CSD)
 *         for AMD MI355X (gfx950).
 *
 * One call of csd_verify is the verification loop of Algorithm 1 for a whole batch at greedy
 * decoding: for each of B sequences, k draft tokens are checked against k+1 rows of vocab-wide
 * target logits.  A draft token is kept when it equals the target's argmax t*, or when it is
 * rescued: the Online Correction Memory holds the ordered pair (draft, t*) with count >= lambda
 * ("Candidate Proposal") AND the Semantic Consistency Gate passes, p(draft)/p(t*) >= tau on the raw
 * logits (Eq. 3).  Every processed divergence increments its pair's count ("Dynamic Update"), rescued
 * or not; positions after the first non-rescued divergence are neither tested nor counted.
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer owned by the caller unless stated otherwise.  The library
 *    allocates nothing, frees nothing and never synchronises: work is enqueued on `stream`
 *    (a hipStream_t passed as void*; NULL = the default stream) and results are valid once the
 *    stream reaches that point.
 *  - Return value: CSD_OK (0) = enqueued; a negative code = argument error detected on the host,
 *    nothing was enqueued and no output was touched.  Conditions that only the device can see
 *    (table full, draft id out of range) are reported through `status`.
 *  - Batches: every memory lookup of a call reads the table as it stood when the call began; the
 *    call's increments are applied after all lookups (kernels of one call are stream-ordered).
 *    Calls that share a table must be ordered on one stream (or by events); concurrent calls on
 *    one table give well-formed counts but unspecified lookup timing.
 */
#ifndef CSD_H
#define CSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* return codes */
#define CSD_OK 0
#define CSD_EINVAL (-1)   /* bad scalar argument or NULL where a pointer is required        */
#define CSD_EALIGN (-2)   /* logits base or row pitch not 16-byte aligned, or outputs misaligned */
#define CSD_ENOSPACE (-3) /* workspace smaller than csd_verify_workspace_bytes()             */
#define CSD_EHIP (-4)     /* a kernel launch was refused by the runtime                      */

/* storage type of the logits */
#define CSD_DTYPE_F32 0
#define CSD_DTYPE_BF16 1

/* csd_verify flags */
#define CSD_APPLY_UPDATES 1u /* apply this call's count increments to the table (Algorithm 1, UpdateMemory) */

/* limits */
#define CSD_MAX_K 63           /* draft tokens per sequence                       */
#define CSD_MAX_V (1u << 20)   /* vocabulary size (token ids fit 20 bits)         */
#define CSD_MAX_SHARDS 8       /* vocabulary shards csd_verify_shards merges       */

/*
 * Online Correction Memory: an open-addressed table of `capacity` (a power of two) 64-bit slots,
 * linear probing, no deletion.  Slot layout (part of the ABI; a table can be copied out and decoded):
 *     bits 63..40  count   (24 bits, saturates at CSD_OCM_COUNT_MAX)
 *     bits 39..20  draft token id
 *     bits 19..0   target token id (t*)
 * The pair is ORDERED: (draft, target) as in T[(x~_i, t*)] of Algorithm 1.  An empty slot holds
 * CSD_OCM_EMPTY (key bits all ones; no counted pair has draft == target, so it is not a valid key).
 * An insert is dropped only when every slot is occupied by another key; the lost increments are
 * added to status[CSD_STATUS_DROPPED].
 */
#define CSD_OCM_KEY_BITS 40
#define CSD_OCM_KEY_MASK 0x000000FFFFFFFFFFull
#define CSD_OCM_EMPTY 0x000000FFFFFFFFFFull
#define CSD_OCM_COUNT_MAX 0xFFFFFFu
#define CSD_OCM_KEY(draft, target) ((((uint64_t)(draft)) << 20) | (uint64_t)(target))

/* status[] indices (uint32 counters, incremented by the kernels, never cleared by the library) */
#define CSD_STATUS_DROPPED 0   /* increments lost because the table was full                     */
#define CSD_STATUS_BAD_DRAFT 1 /* processed draft ids outside [0, V)                             */
#define CSD_STATUS_RESCUED 2   /* positions kept by the memory + gate although draft != t*       */
#define CSD_STATUS_COUNTED 3   /* divergences handed to UpdateMemory                             */
#define CSD_STATUS_ACCEPTED 4   /* draft tokens kept, summed over sequences (acceptance rate = this / (B*k) per call) */
#define CSD_STATUS_STALLED 5   /* waits inside a step that ran out (a GPU starved by other work for seconds): the
                                  sequences concerned report accept_len 0 and next_token -1, their updates are skipped */
#define CSD_STATUS_WORDS 8     /* words 6..7 are reserved and left untouched */

/* pos_flags bits, per draft position; 0 for positions after the stop */
#define CSD_POS_MATCH 1u     /* draft == t*                                        */
#define CSD_POS_FREQ 2u      /* T[(draft,t*)] >= lambda (evaluated on a divergence)  */
#define CSD_POS_SAFE 4u      /* ratio >= tau            (evaluated on a divergence)  */
#define CSD_POS_ACCEPTED 8u  /* position kept                                       */
#define CSD_POS_COUNTED 16u  /* pair handed to UpdateMemory                         */

/*
 * Bytes of device scratch csd_verify needs for this shape (one record per streaming workgroup, the step's
 * rejection log and a small control head).  Returns 0 for invalid arguments.  Host function, no GPU work.
 */
size_t csd_verify_workspace_bytes(int B, int k, int V, int dtype);


/*
 * csd_verify - one verification step for a batch (Algorithm 1, verification loop, temperature 0;
 * Online Correction Memory, phase 2; Semantic Consistency Gating, Eq. 3).
 *
 * Inputs
 *   logits      [B][k+1][V] target logits, row-major, dtype CSD_DTYPE_F32 (float) or CSD_DTYPE_BF16
 *               (bfloat16 bit patterns).  Row r = b*(k+1)+i starts at element r*row_stride.  Values
 *               are finite with |z| <= 2^29 (about 5.4e8), or -inf, with at least one finite value
 *               per row; NaN, +inf and larger magnitudes give undefined results (never a fault).  Base and row pitch must be
 *               16-byte aligned.  Rows 0..k-1 of a sequence belong to its draft positions, row k is
 *               the bonus row.
 *   row_stride  elements between consecutive rows, >= V.
 *   draft       [B][k] draft token ids (int32).  An id outside [0,V) is a divergence with ratio 0 that
 *               is never rescued nor counted; status[CSD_STATUS_BAD_DRAFT] counts processed ones.
 *               May be NULL when k == 0.
 *   tau         gate threshold on p(draft)/p(t*) (inclusive).  tau <= 0: gate always passes;
 *               tau > 1: never passes (strict matching).  NaN is rejected.
 *   lambda      frequency threshold (inclusive).  0: every pair is frequent (gate-only mode).
 *               UINT32_MAX: no pair ever is - plain speculative decoding that still counts its
 *               divergences, i.e. the prior-calibration run that fills the memory before deployment
 *               (Online Correction Memory, phase 1).
 *   ocm         the table, or NULL: no memory (plain strict matching, nothing is updated).
 *   capacity    slots in `ocm`, a power of two >= 1 (ignored when ocm == NULL).
 *   flags       CSD_APPLY_UPDATES or 0.
 * Outputs (written for every sequence / row / position)
 *   accept_len  [B]       n in [0,k]: draft tokens kept.
 *   next_token  [B]       t* of the stopping position, or the argmax of the bonus row when n == k.
 *   argmax      [B][k+1]  t* per row; ties resolve to the lowest token id (float comparison).
 *   row_max     [B][k+1]  max logit (nullable).
 *   row_sumexp  [B][k+1]  sum_v exp(z_v - max); p(t*) = 1/row_sumexp (nullable).
 *   ratio       [B][k]    exp(z[draft] - max) = p(draft)/p(t*) (nullable).
 *   p_draft     [B][k]    ratio / row_sumexp (nullable).
 *   pos_flags   [B][k]    CSD_POS_* bits (nullable).
 *   rej_log     [B][k]    CSD_OCM_KEY(draft, t*) for each counted divergence, CSD_OCM_EMPTY elsewhere
 *                         (nullable; with flags == 0 it can be replayed later through csd_ocm_update).
 *   status      [CSD_STATUS_WORDS] counters, incremented (nullable).
 * A step is ONE kernel launch: workgroups that stream the logits, followed in the same grid by one wave per
 * sequence for the verification logic, which waits for its rows' statistics and then applies the updates
 * (batches of more than 256 sequences use a second launch for the updates).  A step too large to be resident on
 * the GPU at once streams the bonus rows last: the loop, which never reads them, then starts before the stream has
 * ended, and one more wave per sequence takes the bonus row's outputs.  Waits inside the launch are bounded: see
 * CSD_STATUS_STALLED.
 * Scratch
 *   workspace, workspace_bytes   >= csd_verify_workspace_bytes(B,k,V,dtype), 16-byte aligned; needs no
 *                         initialisation and carries nothing from one call to the next (any content will do).
 *                         Two calls in flight must not share a workspace.
 * B == 0 is a valid no-op.  k == 0 verifies nothing and returns the argmax of the single row.
 */
int csd_verify(const void *logits, int dtype, int64_t row_stride, const int32_t *draft, int B, int k, int V, float tau,
               uint32_t lambda, uint64_t *ocm, uint64_t capacity, uint32_t flags, int32_t *accept_len,
               int32_t *next_token, int32_t *argmax, float *row_max, float *row_sumexp, float *ratio, float *p_draft,
               uint8_t *pos_flags, uint64_t *rej_log, uint32_t *status, void *workspace, size_t workspace_bytes,
               void *stream);

/*
 * csd_verify_static - csd_verify for callers that cannot hand over or allocate scratch memory: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, results,
 * kernels and return codes as csd_verify, without `workspace`: the scratch is a CSD_STATIC_SCRATCH_BYTES array
 * inside the library's code object, one copy per GPU, held by every GPU the library runs on until the process
 * ends.  The call allocates and frees nothing; its first use on a device looks the array's device address up
 * once (with that device current - make that first call outside a capture).  `stream` must belong to the
 * current device.
 *   Shapes whose csd_verify_workspace_bytes() exceeds CSD_STATIC_SCRATCH_BYTES return CSD_ENOSPACE (nothing
 *   is enqueued); all five workloads of the benchmark need less than 0.4 MiB.
 *   Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two threads)
 *   race and give undefined results - order them, or use csd_verify with separate workspaces.  The array keeps
 *   the last call's contents; nothing in it has to be cleared between calls.
 */
#define CSD_STATIC_SCRATCH_BYTES (4u << 20)
int csd_verify_static(const void *logits, int dtype, int64_t row_stride, const int32_t *draft, int B, int k, int V, float tau,
                      uint32_t lambda, uint64_t *ocm, uint64_t capacity, uint32_t flags, int32_t *accept_len,
                      int32_t *next_token, int32_t *argmax, float *row_max, float *row_sumexp, float *ratio, float *p_draft,
                      uint8_t *pos_flags, uint64_t *rej_log, uint32_t *status, void *stream);

/*
 * csd_verify_sampled - one verification step at a sampling temperature T > 0 (Algorithm 1 as printed:
 * acceptance test of Eq. 2, correction token from the normalised residual, memory, gate of Eq. 3).  The
 * uniform random numbers the algorithm draws are inputs, so that a run can be reproduced and checked.
 *
 * Per draft position i, with p_i = softmax(target row i / T) and q_i = softmax(draft row i / T):
 *   the draft token is kept when u_accept[b][i] <= min(1, p_i(draft) / q_i(draft));
 *   otherwise t* is drawn from norm(max(0, p_i - q_i)): the smallest token id whose running residual
 *   mass (ascending id) exceeds u_draw[b][i] * (total mass); then T[(draft, t*)] >= lambda and
 *   exp(z(draft) - z(t*)) >= tau on the raw target logits decide the rescue exactly as in csd_verify,
 *   the pair is counted, and the loop stops with t* as the emitted token unless rescued.
 *   When all k tokens are kept the emitted token is drawn from p_{k+1} with u_draw[b][k].
 *
 * Inputs that differ from csd_verify
 *   target_logits [B][k+1][V], draft_logits [B][k][V]   same dtype, each with its own row stride;
 *                 values as for csd_verify, and |z| / T within the same 2^29 bound
 *   temperature   T, 0 < T <= 1e6
 *   u_accept      [B][k] float in [0,1]: the r of the acceptance test
 *   u_draw        [B][k+1] float in [0,1): residual draws of positions 0..k-1, bonus draw at index k
 * Outputs
 *   accept_len [B], next_token [B], pos_flags [B][k] (CSD_POS_MATCH = kept by the acceptance test),
 *   rej_log, status: as for csd_verify
 *   tstar       [B][k]  residual draw of every position whose acceptance test failed (also those the loop
 *                       did not reach), -1 elsewhere (nullable)
 *   bonus_token [B]     the draw from p_{k+1}, computed for every sequence (nullable)
 *   alpha, p_draft, q_draft [B][k]  min(1,p/q), p_i(draft), q_i(draft) at temperature T (nullable)
 *   ratio       [B][k]  exp(z(draft) - z(t*)) where the acceptance test failed, 0 elsewhere (nullable)
 * A draw whose u * mass falls within rounding of a boundary of the running sum may land on either
 * neighbour; a residual without any mass reports the target row's argmax.  An id outside [0,V) ends
 * the loop uncounted with the row's argmax as the emitted token.
 * Three launches: the streaming pass over all 2k+1 rows per sequence, with the acceptance test in waves at the
 * end of the same grid; a second streaming pass over the rows that need a draw (target and draft row side by
 * side); and one launch in which waves invert the running sums while the sequence waves of the same grid wait
 * for their draws and then run the loop with the memory updates.  Waits inside a launch are bounded, see
 * CSD_STATUS_STALLED.
 */
size_t csd_verify_sampled_workspace_bytes(int B, int k, int V, int dtype);
int csd_verify_sampled(const void *target_logits, const void *draft_logits, int dtype, int64_t target_row_stride,
                       int64_t draft_row_stride, const int32_t *draft, int B, int k, int V, float temperature,
                       const float *u_accept, const float *u_draw, float tau, uint32_t lambda, uint64_t *ocm,
                       uint64_t capacity, uint32_t flags, int32_t *accept_len, int32_t *next_token, int32_t *tstar,
                       int32_t *bonus_token, float *alpha, float *p_draft, float *q_draft, float *ratio, uint8_t *pos_flags,
                       uint64_t *rej_log, uint32_t *status, void *workspace, size_t workspace_bytes, void *stream);

/*
 * csd_ocm_update - add counts to the table (UpdateMemory of Algorithm 1 as a separate call; also the
 * bulk load of a calibrated prior, Online Correction Memory phase 1).
 *   keys     [n] CSD_OCM_KEY(draft, target); bits above the key field are ignored; entries equal to
 *            CSD_OCM_EMPTY in the key field are skipped (so a rej_log can be passed as is).
 *   weights  [n] increments (uint32), or NULL = 1 each.  Zero weights are skipped.
 *   n        number of entries (the size of the arrays), 0 is a no-op.
 *   n_dev    NULL, or a DEVICE uint64 holding the number of entries to apply when the call runs: min(n, *n_dev)
 *            are taken.  A list whose length only the device knows - csd_ocm_export's n_out, the reload of a
 *            checkpointed prior, a replica's pairs being folded in - is applied without a host synchronisation,
 *            also from inside a captured graph.
 * Duplicate keys are summed; counts saturate at CSD_OCM_COUNT_MAX; status as for csd_verify (nullable).
 */
int csd_ocm_update(uint64_t *ocm, uint64_t capacity, const uint64_t *keys, const uint32_t *weights, uint64_t n,
                   const uint64_t *n_dev, uint32_t *status, void *stream);

/*
 * csd_ocm_reset - set every slot to CSD_OCM_EMPTY: the empty memory of a run without prior calibration (the
 * starting point of the paper's sensitivity study of online updates alone), and the first step of growing a table.
 */
int csd_ocm_reset(uint64_t *ocm, uint64_t capacity, void *stream);

/*
 * csd_ocm_lookup - read counts: counts[j] = T[keys[j]] (0 if absent).  The "Candidate Proposal" read
 * as a stand-alone call, for inspection and tests.
 */
int csd_ocm_lookup(const uint64_t *ocm, uint64_t capacity, const uint64_t *keys, uint32_t *counts, uint64_t n,
                   void *stream);

/*
 * csd_ocm_merge - T_dst[pair] += T_src[pair] for every pair held by src (counts saturate).  The life cycle
 * of the memory beyond a single run ("prior calibration" is a one-time offline product that later runs
 * start from): growing a table (reset a larger one, merge the old one into it = rehash), combining
 * memories calibrated on different corpora, folding per-device replicas.  dst and src must not overlap.
 * A pair that finds no free slot in dst is dropped and its count added to status[CSD_STATUS_DROPPED].
 */
int csd_ocm_merge(uint64_t *dst, uint64_t dst_capacity, const uint64_t *src, uint64_t src_capacity, uint32_t *status,
                  void *stream);

/*
 * csd_ocm_export - the table as a compact list, layout-independent.  Prior calibration (Online Correction
 * Memory, phase 1) is a one-time, offline product that deployments start from: this is the form it is kept in
 * (a checkpoint) or sent in (between devices): keys_out[j] = CSD_OCM_KEY(draft, target), counts_out[j] = its count, for the
 * n pairs the table holds, in unspecified order.  *n_out (device, uint64) receives n; when n exceeds
 * max_entries only max_entries pairs are written.  keys_out / counts_out may be NULL with max_entries == 0
 * (count only).  The list can be fed back through csd_ocm_update(keys, counts).
 */
int csd_ocm_export(const uint64_t *ocm, uint64_t capacity, uint64_t *keys_out, uint32_t *counts_out, uint64_t max_entries,
                   uint64_t *n_out, void *stream);

/*
 * Row partials: the streaming pass over the logits on its own (the p_{1:gamma+1}(.) statistics of
 * Algorithm 1 before any verification logic).  A row is cut into shares, one per wave (a wave's share is a
 * strided subset of a run of 32 KiB tiles, not a contiguous range of tokens); each wave leaves one
 * csd_row_partial for its share.  A row's statistics follow from its partials as
 *     m  = max_j m_j
 *     t* = min{ idx_j : m_j == m }                       (float comparison)
 *     S  = sum_j s_j * 2^(cref_j - m * CSD_LOG2E_F32)    (skip partials with s_j == 0)
 * where CSD_LOG2E_F32 is log2(e) rounded to float, the constant the kernel multiplies logits by.
 * The same combine merges vocabulary shards of a tensor-parallel LM head (offset idx by the shard base).
 * csd_verify runs exactly this kernel as its first stage.
 */
typedef struct csd_row_partial {
    float m;     /* maximum of the share, -inf if it holds no finite logit            */
    float cref;  /* reference exponent (log2 units) that s is scaled by                */
    float s;     /* sum over the share of 2^(z * CSD_LOG2E_F32 - cref)                 */
    int32_t idx; /* lowest token id in the share whose logit equals m                  */
} csd_row_partial;
#define CSD_LOG2E_F32 1.4426950408889634f

/* Partials per row that csd_row_partials writes for `rows` rows of V logits (0 = invalid shape). Host only. */
int csd_row_partials_per_row(int rows, int V, int dtype);

/*
 * csd_row_partials - enqueue the streaming pass: partials[r * per_row + j], j < per_row, for r < rows.
 *   logits, dtype, row_stride, V   as for csd_verify (rows are [rows][V], 16-byte aligned pitch)
 *   partials                      device buffer of rows * csd_row_partials_per_row(rows,V,dtype) entries,
 *                                 16-byte aligned; partials_bytes is its size (CSD_ENOSPACE if too small)
 */
int csd_row_partials(const void *logits, int dtype, int64_t row_stride, int rows, int V, csd_row_partial *partials,
                     size_t partials_bytes, void *stream);

/*
 * Vocabulary shards.  When the target's logits exist only as shards of the vocabulary - a tensor-parallel
 * LM head (Implementation Details: each 70B-class target spans two devices), or a head evaluated chunk by
 * chunk - each shard runs
 * csd_row_partials on its [B*(k+1)][V_s] slice and csd_shard_draft_logits to pick out the logits of the
 * draft tokens it owns; the partials (16 bytes each) and the [B][k] draft logits are all that has to be
 * brought together, and csd_verify_shards does the rest of the step from them: the same combine, lookup,
 * gate, scan and updates as csd_verify, with token ids of shard s offset by shard_base[s].
 *
 * csd_shard_draft_logits: draft_logit[b][i] = logits[b][i][draft[b][i] - base] where base <= draft[b][i] <
 *   base + V_shard; other entries are left untouched (so shards on one device can share the buffer, and
 *   buffers of several devices merge by taking, per entry, the one value that was written).
 * csd_verify_shards:
 *   n_shards (1..CSD_MAX_SHARDS); shard_partials, shard_per_row, shard_base: HOST arrays of n_shards entries
 *     (device pointer to the shard's partials [B*(k+1)][shard_per_row[s]], its partials per row as
 *     csd_row_partials_per_row reported, the token id of its first logit)
 *   draft_logit [B][k] device; V = the whole vocabulary; everything else as csd_verify.
 *   workspace >= csd_verify_shards_workspace_bytes(B, k).
 */
size_t csd_verify_shards_workspace_bytes(int B, int k);
int csd_verify_shards(int n_shards, const csd_row_partial *const *shard_partials, const int *shard_per_row,
                      const int *shard_base, const float *draft_logit, const int32_t *draft, int B, int k, int V, float tau,
                      uint32_t lambda, uint64_t *ocm, uint64_t capacity, uint32_t flags, int32_t *accept_len,
                      int32_t *next_token, int32_t *argmax, float *row_max, float *row_sumexp, float *ratio, float *p_draft,
                      uint8_t *pos_flags, uint64_t *rej_log, uint32_t *status, void *workspace, size_t workspace_bytes,
                      void *stream);
int csd_shard_draft_logits(const void *logits, int dtype, int64_t row_stride, int B, int k, int V_shard, int base,
                           const int32_t *draft, float *draft_logit, void *stream);

/* Static string for a return code (host pointer, never NULL). */
const char *csd_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CSD_H */
