// C ABI of the CSD verification library: argument validation and kernel sequencing.
// Nothing here allocates, frees or synchronises; every entry point only enqueues on the caller's stream.
#include <atomic>
#include <chrono>
#include <cstring>

#include "csd_internal.h"

namespace csd {
namespace {

bool shape_ok(int B, int k, int V, int dtype) {
    if (B < 0 || k < 0 || k > CSD_MAX_K) return false;
    if (V < 1 || (uint32_t)V > CSD_MAX_V) return false;
    if (dtype != CSD_DTYPE_F32 && dtype != CSD_DTYPE_BF16) return false;
    if ((int64_t)B * (k + 1) > (int64_t)1 << 24) return false;   // keeps every grid and index within 31 bits
    return true;
}

bool is_nan_bits(float f) {   // bit test: independent of the floating-point options of the build
    uint32_t u;
    std::memcpy(&u, &f, sizeof u);
    return (u & 0x7FFFFFFFu) > 0x7F800000u;
}
constexpr uint64_t kMaxInKernelUpdates = 8192;   // log entries one wave applies at the end of the finish kernel

bool is_pow2(uint64_t x) { return x != 0 && (x & (x - 1)) == 0; }
bool aligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

}  // namespace
}  // namespace csd

using namespace csd;

// Scratch of csd_verify_static: one copy per GPU, loaded with the code object and held until the process ends.
// The name below is a host-side stand-in, not a device address: host code only ever uses the pointer that
// hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[CSD_STATIC_SCRATCH_BYTES];

namespace {
// A number that differs from call to call (and, by its starting point, from process to process): the records
// that the waves of a step hand to each other are tagged with it, so what an earlier call left in a workspace
// never passes for this call's.
uint64_t next_call_number() {
    static std::atomic<uint64_t> counter{[] {
        uint64_t x = (uint64_t)std::chrono::steady_clock::now().time_since_epoch().count();
        x ^= (uint64_t)(uintptr_t)&x * 0x9E3779B97F4A7C15ull;
        return x | 1ull;
    }()};
    return counter.fetch_add(0x9E3779B97F4A7C15ull, std::memory_order_relaxed);
}

// Test hooks (csd_test_set_wait_rules, not part of csd.h): how long waits inside a launch may last, and a mask
// that makes the readers' per-call number differ from the writers' so that nothing ever passes - the way to see,
// without ever hanging a kernel, that a wait that runs out is reported and leaves everything consistent.
std::atomic<uint32_t> g_spin_limit{1u << 21};
std::atomic<uint64_t> g_reader_nonce_xor{0};

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device; looked up once per device (no allocation), nullptr on error.
void *static_scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p != nullptr) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return nullptr;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}
}  // namespace

// One greedy verification step on the given scratch memory: validation, then the two (or three) launches.
static int verify_step(const void *logits, int dtype, int64_t row_stride, const int32_t *draft, int B, int k, int V, float tau,
                       uint32_t lambda, uint64_t *ocm, uint64_t capacity, uint32_t flags, int32_t *accept_len,
                       int32_t *next_token, int32_t *argmax, float *row_max, float *row_sumexp, float *ratio, float *p_draft,
                       uint8_t *pos_flags, uint64_t *rej_log, uint32_t *status, void *workspace, size_t workspace_bytes,
                       void *stream) {
    if (!shape_ok(B, k, V, dtype)) return CSD_EINVAL;
    if (is_nan_bits(tau)) return CSD_EINVAL;
    if (flags & ~CSD_APPLY_UPDATES) return CSD_EINVAL;
    if (B == 0) return CSD_OK;
    if (!logits || !accept_len || !next_token || !argmax || !workspace) return CSD_EINVAL;
    if (k > 0 && !draft) return CSD_EINVAL;
    if (row_stride < V) return CSD_EINVAL;
    if (ocm && !is_pow2(capacity)) return CSD_EINVAL;
    const size_t esz = (dtype == CSD_DTYPE_F32) ? 4 : 2;
    if (!aligned(logits, 16) || ((size_t)row_stride * esz) % 16 != 0) return CSD_EALIGN;
    if (!aligned(workspace, 16) || !aligned(accept_len, 4) || !aligned(next_token, 4) || !aligned(argmax, 4) ||
        !aligned(draft, 4) || !aligned(row_max, 4) || !aligned(row_sumexp, 4) || !aligned(ratio, 4) ||
        !aligned(p_draft, 4) || !aligned(rej_log, 8) || !aligned(ocm, 8) || !aligned(status, 4))
        return CSD_EALIGN;

    const StreamPlan plan = make_stream_plan(B * (k + 1), V, dtype);
    const WorkspaceLayout ws = make_workspace_layout(plan, B, k);
    if (workspace_bytes < ws.total) return CSD_ENOSPACE;

    hipStream_t st = (hipStream_t)stream;
    const bool apply = (flags & CSD_APPLY_UPDATES) && ocm != nullptr && k > 0;
    uint64_t *log = rej_log ? rej_log : (apply ? (uint64_t *)((char *)workspace + ws.log_off) : nullptr);

    EpilogueArgs a = {};
    a.logits = logits;
    a.dtype = dtype;
    a.row_stride = row_stride;
    a.draft = draft;
    a.B = B;
    a.k = k;
    a.V = V;
    a.tau = tau;
    a.lambda = lambda;
    a.ocm = ocm;
    a.capacity = capacity;
    a.sharded = 0;
    a.n_shards = 1;
    a.shard_partials[0] = nullptr;                        // the records of the single-launch step take their place
    a.shard_per_row[0] = plan.nsplit;                     // one record per streaming workgroup
    a.shard_base[0] = 0;
    a.draft_logit = nullptr;
    a.accept_len = accept_len;
    a.next_token = next_token;
    a.argmax = argmax;
    a.row_max = row_max;
    a.row_sumexp = row_sumexp;
    a.ratio = ratio;
    a.p_draft = p_draft;
    a.pos_flags = pos_flags;
    a.rej_log = log;
    a.status = status;
    a.batch_ticket = nullptr;
    // One launch does the whole step.  The step's increments are applied inside it by the sequence waves
    // themselves while their workgroups are few enough to wait for each other; larger batches hand the log to
    // the bulk update kernel (one more launch, many workgroups).
    const int n_seq_wgs = (B + kStepSeqWaves - 1) / kStepSeqWaves;
    const bool update_here = apply && n_seq_wgs <= kMaxBarrierWorkgroups;
    a.apply_updates = update_here ? 1 : 0;
    a.update_here = update_here ? 1 : 0;
    if (update_here && !rej_log) a.rej_log = nullptr;      // nobody reads a log then
    a.records = (StepRecord *)((char *)workspace + ws.partials_off);
    a.ctrl = (StepControl *)((char *)workspace + ws.ticket_off);
    a.nonce = next_call_number();
    a.reader_nonce = a.nonce ^ g_reader_nonce_xor.load(std::memory_order_relaxed);
    a.spin_limit = g_spin_limit.load(std::memory_order_relaxed);
    a.n_stream_wgs = plan.rows * plan.nsplit;
    a.n_seq_wgs = n_seq_wgs;
    a.order = make_step_order(plan, B, k);
    a.seq_words = (WordRecord *)((char *)workspace + ws.words_off);
    const StreamSource src = {(const char *)logits, row_stride * (int64_t)esz, plan.rows, nullptr, 0, CSD_LOG2E_F32};
    if (launch_verify_step(src, dtype, V, plan, a, st) != hipSuccess) return CSD_EHIP;
    if (apply && !update_here) {
        if (launch_ocm_update(ocm, capacity, log, nullptr, (uint64_t)B * (uint64_t)k, nullptr, status, st) != hipSuccess) return CSD_EHIP;
    }
    return CSD_OK;
}


extern "C" {

size_t csd_verify_workspace_bytes(int B, int k, int V, int dtype) {
    if (!shape_ok(B, k, V, dtype)) return 0;
    const StreamPlan p = make_stream_plan(B * (k + 1), V, dtype);
    return make_workspace_layout(p, B, k).total;
}

int csd_verify(const void *logits, int dtype, int64_t row_stride, const int32_t *draft, int B, int k, int V, float tau,
               uint32_t lambda, uint64_t *ocm, uint64_t capacity, uint32_t flags, int32_t *accept_len,
               int32_t *next_token, int32_t *argmax, float *row_max, float *row_sumexp, float *ratio, float *p_draft,
               uint8_t *pos_flags, uint64_t *rej_log, uint32_t *status, void *workspace, size_t workspace_bytes,
               void *stream) {
    return verify_step(logits, dtype, row_stride, draft, B, k, V, tau, lambda, ocm, capacity, flags, accept_len, next_token,
                       argmax, row_max, row_sumexp, ratio, p_draft, pos_flags, rej_log, status, workspace, workspace_bytes,
                       stream);
}

int csd_verify_static(const void *logits, int dtype, int64_t row_stride, const int32_t *draft, int B, int k, int V, float tau,
                      uint32_t lambda, uint64_t *ocm, uint64_t capacity, uint32_t flags, int32_t *accept_len,
                      int32_t *next_token, int32_t *argmax, float *row_max, float *row_sumexp, float *ratio, float *p_draft,
                      uint8_t *pos_flags, uint64_t *rej_log, uint32_t *status, void *stream) {
    if (!shape_ok(B, k, V, dtype)) return CSD_EINVAL;
    if (csd_verify_workspace_bytes(B, k, V, dtype) > (size_t)CSD_STATIC_SCRATCH_BYTES) return CSD_ENOSPACE;
    void *ws = static_scratch_of_current_device();
    if (ws == nullptr) return CSD_EHIP;
    return verify_step(logits, dtype, row_stride, draft, B, k, V, tau, lambda, ocm, capacity, flags, accept_len, next_token,
                       argmax, row_max, row_sumexp, ratio, p_draft, pos_flags, rej_log, status, ws, CSD_STATIC_SCRATCH_BYTES,
                       stream);
}

size_t csd_verify_shards_workspace_bytes(int B, int k) {
    if (B < 0 || k < 0 || k > CSD_MAX_K || (int64_t)B * (k + 1) > (int64_t)1 << 24) return 0;
    return 256 + (((size_t)B * (size_t)k * sizeof(uint64_t) + 255) & ~(size_t)255);
}

int csd_verify_shards(int n_shards, const csd_row_partial *const *shard_partials, const int *shard_per_row,
                      const int *shard_base, const float *draft_logit, const int32_t *draft, int B, int k, int V, float tau,
                      uint32_t lambda, uint64_t *ocm, uint64_t capacity, uint32_t flags, int32_t *accept_len,
                      int32_t *next_token, int32_t *argmax, float *row_max, float *row_sumexp, float *ratio, float *p_draft,
                      uint8_t *pos_flags, uint64_t *rej_log, uint32_t *status, void *workspace, size_t workspace_bytes,
                      void *stream) {
    if (!shape_ok(B, k, V, CSD_DTYPE_F32)) return CSD_EINVAL;
    if (n_shards < 1 || n_shards > CSD_MAX_SHARDS || !shard_partials || !shard_per_row || !shard_base) return CSD_EINVAL;
    if (is_nan_bits(tau) || (flags & ~CSD_APPLY_UPDATES)) return CSD_EINVAL;
    if (B == 0) return CSD_OK;
    if (!accept_len || !next_token || !argmax || !workspace) return CSD_EINVAL;
    if (k > 0 && (!draft || !draft_logit)) return CSD_EINVAL;
    if (ocm && !is_pow2(capacity)) return CSD_EINVAL;
    for (int s = 0; s < n_shards; ++s) {
        if (!shard_partials[s] || shard_per_row[s] < 1 || shard_base[s] < 0 || shard_base[s] >= V) return CSD_EINVAL;
        if (!aligned(shard_partials[s], 16)) return CSD_EALIGN;
    }
    if (!aligned(workspace, 16) || !aligned(accept_len, 4) || !aligned(next_token, 4) || !aligned(argmax, 4) ||
        !aligned(draft, 4) || !aligned(draft_logit, 4) || !aligned(row_max, 4) || !aligned(row_sumexp, 4) ||
        !aligned(ratio, 4) || !aligned(p_draft, 4) || !aligned(rej_log, 8) || !aligned(ocm, 8) || !aligned(status, 4))
        return CSD_EALIGN;
    if (workspace_bytes < csd_verify_shards_workspace_bytes(B, k)) return CSD_ENOSPACE;

    hipStream_t st = (hipStream_t)stream;
    const bool apply = (flags & CSD_APPLY_UPDATES) && ocm != nullptr && k > 0;
    EpilogueArgs a = {};
    a.logits = nullptr;
    a.dtype = CSD_DTYPE_F32;
    a.row_stride = 0;
    a.draft = draft;
    a.B = B;
    a.k = k;
    a.V = V;
    a.tau = tau;
    a.lambda = lambda;
    a.ocm = ocm;
    a.capacity = capacity;
    a.sharded = 1;
    a.n_shards = n_shards;
    for (int s = 0; s < n_shards; ++s) {
        a.shard_partials[s] = shard_partials[s];
        a.shard_per_row[s] = shard_per_row[s];
        a.shard_base[s] = shard_base[s];
    }
    a.draft_logit = draft_logit;
    a.accept_len = accept_len;
    a.next_token = next_token;
    a.argmax = argmax;
    a.row_max = row_max;
    a.row_sumexp = row_sumexp;
    a.ratio = ratio;
    a.p_draft = p_draft;
    a.pos_flags = pos_flags;
    a.rej_log = rej_log ? rej_log : (apply ? (uint64_t *)((char *)workspace + 256) : nullptr);
    a.status = status;
    a.batch_ticket = (uint32_t *)workspace;
    const bool update_in_finish = apply && (uint64_t)B * (uint64_t)k <= kMaxInKernelUpdates;
    a.apply_updates = update_in_finish ? 1 : 0;
    if (update_in_finish && launch_zero_ticket(a.batch_ticket, st) != hipSuccess) return CSD_EHIP;
    if (launch_finish(a, st) != hipSuccess) return CSD_EHIP;
    if (apply && !update_in_finish) {
        if (launch_ocm_update(ocm, capacity, a.rej_log, nullptr, (uint64_t)B * (uint64_t)k, nullptr, status, st) != hipSuccess)
            return CSD_EHIP;
    }
    return CSD_OK;
}

int csd_shard_draft_logits(const void *logits, int dtype, int64_t row_stride, int B, int k, int V_shard, int base,
                           const int32_t *draft, float *draft_logit, void *stream) {
    if (!shape_ok(B, k, V_shard, dtype) || base < 0 || (int64_t)base + V_shard > (int64_t)CSD_MAX_V) return CSD_EINVAL;
    if (B == 0 || k == 0) return CSD_OK;
    if (!logits || !draft || !draft_logit || row_stride < V_shard) return CSD_EINVAL;
    const size_t esz = (dtype == CSD_DTYPE_F32) ? 4 : 2;
    if (!aligned(logits, esz) || !aligned(draft, 4) || !aligned(draft_logit, 4)) return CSD_EALIGN;
    return launch_shard_draft_logits(logits, dtype, row_stride, B, k, V_shard, base, draft, draft_logit,
                                     (hipStream_t)stream) == hipSuccess ? CSD_OK : CSD_EHIP;
}

static SampledWorkspace sampled_layout(const StreamPlan &plan, int B, int k, int nseg) {
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    SampledWorkspace w;
    const size_t K1 = (size_t)k + 1;
    w.ticket_off = 0;
    w.partials_off = 256;
    w.rows_off = up(w.partials_off + (size_t)plan.rows * plan.nsplit * sizeof(StepRecord));   // one record per streaming workgroup
    w.work_off = up(w.rows_off + (size_t)B * K1 * sizeof(DrawRow));
    w.segsum_off = up(w.work_off + (size_t)B * K1 * sizeof(int32_t));
    w.zpd_off = up(w.segsum_off + (size_t)B * K1 * (size_t)nseg * sizeof(float));
    w.state_off = up(w.zpd_off + (size_t)B * k * sizeof(float));
    w.tstar_off = up(w.state_off + (size_t)B * k);
    w.bonus_off = up(w.tstar_off + (size_t)B * k * sizeof(int32_t));
    w.draws_off = up(w.bonus_off + (size_t)B * sizeof(int32_t));
    w.log_off = up(w.draws_off + (size_t)B * K1 * sizeof(WordRecord));
    w.total = up(w.log_off + (size_t)B * k * sizeof(uint64_t));
    return w;
}

size_t csd_verify_sampled_workspace_bytes(int B, int k, int V, int dtype) {
    if (!shape_ok(B, k, V, dtype)) return 0;
    if ((int64_t)B * (2 * k + 1) > (int64_t)1 << 24) return 0;
    const StreamPlan p = make_stream_plan(B * (2 * k + 1), V, dtype);
    return sampled_layout(p, B, k, sampled_segments(V, dtype)).total;
}

int csd_verify_sampled(const void *target_logits, const void *draft_logits, int dtype, int64_t target_row_stride,
                       int64_t draft_row_stride, const int32_t *draft, int B, int k, int V, float temperature,
                       const float *u_accept, const float *u_draw, float tau, uint32_t lambda, uint64_t *ocm,
                       uint64_t capacity, uint32_t flags, int32_t *accept_len, int32_t *next_token, int32_t *tstar,
                       int32_t *bonus_token, float *alpha, float *p_draft, float *q_draft, float *ratio, uint8_t *pos_flags,
                       uint64_t *rej_log, uint32_t *status, void *workspace, size_t workspace_bytes, void *stream) {
    if (!shape_ok(B, k, V, dtype) || (int64_t)B * (2 * k + 1) > (int64_t)1 << 24) return CSD_EINVAL;
    if (is_nan_bits(tau) || is_nan_bits(temperature) || !(temperature > 0.f) || temperature > 1e6f) return CSD_EINVAL;
    const float scale = (float)(1.4426950408889634 / (double)temperature);
    if (!(scale > 1e-6f) || !(scale < 1e6f)) return CSD_EINVAL;
    if (flags & ~CSD_APPLY_UPDATES) return CSD_EINVAL;
    if (B == 0) return CSD_OK;
    if (!target_logits || !accept_len || !next_token || !workspace || !u_draw) return CSD_EINVAL;
    if (k > 0 && (!draft || !draft_logits || !u_accept)) return CSD_EINVAL;
    if (target_row_stride < V || (k > 0 && draft_row_stride < V)) return CSD_EINVAL;
    if (ocm && !is_pow2(capacity)) return CSD_EINVAL;
    const size_t esz = (dtype == CSD_DTYPE_F32) ? 4 : 2;
    if (!aligned(target_logits, 16) || ((size_t)target_row_stride * esz) % 16 != 0) return CSD_EALIGN;
    if (k > 0 && (!aligned(draft_logits, 16) || ((size_t)draft_row_stride * esz) % 16 != 0)) return CSD_EALIGN;
    if (!aligned(workspace, 16) || !aligned(accept_len, 4) || !aligned(next_token, 4) || !aligned(tstar, 4) ||
        !aligned(bonus_token, 4) || !aligned(draft, 4) || !aligned(u_accept, 4) || !aligned(u_draw, 4) || !aligned(alpha, 4) ||
        !aligned(p_draft, 4) || !aligned(q_draft, 4) || !aligned(ratio, 4) || !aligned(rej_log, 8) || !aligned(ocm, 8) ||
        !aligned(status, 4))
        return CSD_EALIGN;

    const int rows_p = B * (k + 1), rows_q = B * k;
    const StreamPlan plan = make_stream_plan(rows_p + rows_q, V, dtype);
    const int nseg = sampled_segments(V, dtype);
    const SampledWorkspace ws = sampled_layout(plan, B, k, nseg);
    if (workspace_bytes < ws.total) return CSD_ENOSPACE;
    char *wsp = (char *)workspace;
    hipStream_t st = (hipStream_t)stream;
    const bool apply = (flags & CSD_APPLY_UPDATES) && ocm != nullptr && k > 0;

    SampledArgs a;
    a.target = target_logits;
    a.draft_logits = draft_logits;
    a.dtype = dtype;
    a.target_stride = target_row_stride;
    a.draft_stride = draft_row_stride;
    a.draft = draft;
    a.B = B;
    a.k = k;
    a.V = V;
    a.scale = scale;
    a.u_accept = u_accept;
    a.u_draw = u_draw;
    a.tau = tau;
    a.lambda = lambda;
    a.ocm = ocm;
    a.capacity = capacity;
    a.records = (StepRecord *)(wsp + ws.partials_off);
    a.nsplit = plan.nsplit;
    a.n_stream_wgs = plan.rows * plan.nsplit;
    a.nseg = nseg;
    a.rows = (DrawRow *)(wsp + ws.rows_off);
    a.list_ctrl = (StepControl *)(wsp + ws.ticket_off);
    a.work_rows = (int32_t *)(wsp + ws.work_off);
    a.segsum = (float *)(wsp + ws.segsum_off);
    a.pos_zpd = (float *)(wsp + ws.zpd_off);
    a.pos_state = (uint8_t *)(wsp + ws.state_off);
    a.tstar = tstar ? tstar : (int32_t *)(wsp + ws.tstar_off);
    a.bonus = bonus_token ? bonus_token : (int32_t *)(wsp + ws.bonus_off);
    a.accept_len = accept_len;
    a.next_token = next_token;
    a.alpha = alpha;
    a.p_draft = p_draft;
    a.q_draft = q_draft;
    a.ratio = ratio;
    a.pos_flags = pos_flags;
    a.rej_log = rej_log ? rej_log : (apply ? (uint64_t *)(wsp + ws.log_off) : nullptr);
    a.status = status;
    a.draws = (WordRecord *)(wsp + ws.draws_off);
    a.ctrl = (StepControl *)(wsp + ws.ticket_off + sizeof(StepControl));   // behind the list's control head
    a.nonce = next_call_number();
    a.reader_nonce = a.nonce ^ g_reader_nonce_xor.load(std::memory_order_relaxed);
    a.spin_limit = g_spin_limit.load(std::memory_order_relaxed);
    a.n_loc_wgs = sampled_locate_workgroups(B, k);
    // as in csd_verify: few sequence workgroups wait for each other and apply the updates themselves, many hand the
    // log to the bulk update kernel
    const bool update_in_tail = apply && sampled_sequence_workgroups(B) <= kMaxBarrierWorkgroups;
    a.update_here = update_in_tail ? 1 : 0;
    if (update_in_tail && !rej_log) a.rej_log = nullptr;   // nobody reads a log then

    const StreamSource src = {(const char *)target_logits, target_row_stride * (int64_t)esz, rows_p,
                              (const char *)draft_logits, draft_row_stride * (int64_t)esz, scale};
    if (launch_sampled_step(src, a, st) != hipSuccess) return CSD_EHIP;
    if (apply && !update_in_tail) {
        if (launch_ocm_update(ocm, capacity, a.rej_log, nullptr, (uint64_t)B * (uint64_t)k, nullptr, status, st) != hipSuccess)
            return CSD_EHIP;
    }
    return CSD_OK;
}

int csd_ocm_update(uint64_t *ocm, uint64_t capacity, const uint64_t *keys, const uint32_t *weights, uint64_t n,
                   const uint64_t *n_dev, uint32_t *status, void *stream) {
    if (!ocm || !is_pow2(capacity)) return CSD_EINVAL;
    if (n == 0) return CSD_OK;
    if (!keys || n > ((uint64_t)1 << 40)) return CSD_EINVAL;
    if (!aligned(ocm, 8) || !aligned(keys, 8) || !aligned(weights, 4) || !aligned(n_dev, 8) || !aligned(status, 4)) return CSD_EALIGN;
    return launch_ocm_update(ocm, capacity, keys, weights, n, n_dev, status, (hipStream_t)stream) == hipSuccess ? CSD_OK : CSD_EHIP;
}

int csd_ocm_reset(uint64_t *ocm, uint64_t capacity, void *stream) {
    if (!ocm || !is_pow2(capacity)) return CSD_EINVAL;
    if (!aligned(ocm, 8)) return CSD_EALIGN;
    return launch_ocm_reset(ocm, capacity, (hipStream_t)stream) == hipSuccess ? CSD_OK : CSD_EHIP;
}

int csd_ocm_lookup(const uint64_t *ocm, uint64_t capacity, const uint64_t *keys, uint32_t *counts, uint64_t n,
                   void *stream) {
    if (!ocm || !is_pow2(capacity)) return CSD_EINVAL;
    if (n == 0) return CSD_OK;
    if (!keys || !counts) return CSD_EINVAL;
    if (!aligned(ocm, 8) || !aligned(keys, 8) || !aligned(counts, 4)) return CSD_EALIGN;
    return launch_ocm_lookup(ocm, capacity, keys, counts, n, (hipStream_t)stream) == hipSuccess ? CSD_OK : CSD_EHIP;
}

int csd_ocm_merge(uint64_t *dst, uint64_t dst_capacity, const uint64_t *src, uint64_t src_capacity, uint32_t *status,
                  void *stream) {
    if (!dst || !src || !is_pow2(dst_capacity) || !is_pow2(src_capacity)) return CSD_EINVAL;
    if (!aligned(dst, 8) || !aligned(src, 8) || !aligned(status, 4)) return CSD_EALIGN;
    const uintptr_t d0 = (uintptr_t)dst, d1 = d0 + dst_capacity * 8, s0 = (uintptr_t)src, s1 = s0 + src_capacity * 8;
    if (d0 < s1 && s0 < d1) return CSD_EINVAL;   // overlapping tables
    return launch_ocm_merge(dst, dst_capacity, src, src_capacity, status, (hipStream_t)stream) == hipSuccess ? CSD_OK : CSD_EHIP;
}

int csd_ocm_export(const uint64_t *ocm, uint64_t capacity, uint64_t *keys_out, uint32_t *counts_out, uint64_t max_entries,
                   uint64_t *n_out, void *stream) {
    if (!ocm || !is_pow2(capacity) || !n_out) return CSD_EINVAL;
    if (max_entries > 0 && (!keys_out || !counts_out)) return CSD_EINVAL;
    if (!aligned(ocm, 8) || !aligned(keys_out, 8) || !aligned(counts_out, 4) || !aligned(n_out, 8)) return CSD_EALIGN;
    return launch_ocm_export(ocm, capacity, keys_out, counts_out, max_entries, n_out, (hipStream_t)stream) == hipSuccess
               ? CSD_OK : CSD_EHIP;
}

int csd_row_partials_per_row(int rows, int V, int dtype) {
    if (rows < 0 || !shape_ok(0, 0, V, dtype) || rows > (1 << 24)) return 0;
    return make_stream_plan(rows, V, dtype).partials_per_row;
}

int csd_row_partials(const void *logits, int dtype, int64_t row_stride, int rows, int V, csd_row_partial *partials,
                     size_t partials_bytes, void *stream) {
    if (rows < 0 || rows > (1 << 24) || !shape_ok(0, 0, V, dtype)) return CSD_EINVAL;
    if (rows == 0) return CSD_OK;
    if (!logits || !partials || row_stride < V) return CSD_EINVAL;
    const size_t esz = (dtype == CSD_DTYPE_F32) ? 4 : 2;
    if (!aligned(logits, 16) || ((size_t)row_stride * esz) % 16 != 0 || !aligned(partials, 16)) return CSD_EALIGN;
    const StreamPlan plan = make_stream_plan(rows, V, dtype);
    if (partials_bytes < (size_t)rows * plan.partials_per_row * sizeof(RowPartial)) return CSD_ENOSPACE;
    const StreamSource src = {(const char *)logits, row_stride * (int64_t)esz, rows, nullptr, 0, CSD_LOG2E_F32};
    return launch_row_partials(src, dtype, V, plan, partials, (hipStream_t)stream) == hipSuccess ? CSD_OK : CSD_EHIP;
}

// Test hook, deliberately absent from csd.h: spin_limit = polls a wait inside a launch may take (0 restores the
// default), reader_nonce_xor != 0 makes every such wait run out.  Affects calls enqueued afterwards.
void csd_test_set_wait_rules(uint32_t spin_limit, uint64_t reader_nonce_xor) {
    g_spin_limit.store(spin_limit ? spin_limit : (1u << 21), std::memory_order_relaxed);
    g_reader_nonce_xor.store(reader_nonce_xor, std::memory_order_relaxed);
}

// Test hook, deliberately absent from csd.h: the grid order of csd_verify's launch - 0 chosen by shape (the default),
// 1 always the plain order, 2 the bonus rows last whenever there is a draft position.  Affects calls enqueued afterwards.
void csd_test_set_step_order(int order) { set_step_order_override(order); }
// 1 when csd_verify streams the bonus rows of this shape last, 0 for the plain order, -1 for a bad shape (host arithmetic)
int csd_test_step_order_of(int B, int k, int V, int dtype) {
    if (!shape_ok(B, k, V, dtype)) return -1;
    return make_step_order(make_stream_plan(B * (k + 1), V, dtype), B, k).bonus_last;
}

const char *csd_strerror(int code) {
    switch (code) {
        case CSD_OK: return "ok";
        case CSD_EINVAL: return "invalid argument";
        case CSD_EALIGN: return "misaligned pointer or row pitch";
        case CSD_ENOSPACE: return "workspace too small";
        case CSD_EHIP: return "kernel launch failed";
        default: return "unknown csd error";
    }
}

}  // extern "C"
