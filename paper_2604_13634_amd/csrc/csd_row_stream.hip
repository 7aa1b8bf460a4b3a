// Row-stream kernel: the one pass over the vocab-wide target logits.
//
// For every verify row (a draft position or the bonus row of Algorithm 1) the verification step
// needs the target distribution's normaliser, the greedy target token t* and, later, single
// probabilities (Eq. 3 and the p_i(.) of Algorithm 1):
//     m = max_v z_v,   t* = min{v : z_v == m},   S = sum_v exp(z_v - m).
// This is a pure streaming reduction: every logit is read from HBM exactly once with 16-byte
// loads, nothing is reused, so the kernel is bound by HBM bandwidth (no MFMA, no LDS staging).
//
// Work split: a row is cut into `nsplit` segments of whole tiles; a workgroup of 4 waves owns one
// (row, segment) and its waves interleave 1 KiB wave-loads so the group walks contiguous memory.
// Each wave keeps its own running state and writes one RowPartial; there is no cross-wave step
// here - the per-sequence epilogue combines the partials of a row in double precision.
//
// Per-lane running state (fp32):
//   rm      running maximum;  best_it = iteration at which rm last strictly increased, i.e. the
//           first 16-byte chunk of this lane that holds the value rm (lanes visit chunks in
//           ascending address order, so "first" is "lowest token id").
//   s[E]    sums of 2^(z*log2e - c), one per element slot of a chunk, against a WAVE-UNIFORM
//           reference exponent c.  c is not the running maximum: it is only kept within kRescaleGap
//           of it, which is all that floating point needs (no overflow, full relative precision).
//           A rescale (wave reduction + multiply) happens only when some lane's maximum climbs more
//           than kRescaleGap above the reference - the first iteration, then almost never - so the
//           steady-state loop is unpack, max3, fma, v_exp_f32, add and one compare per tile.
// The exponent error of a term is half an ulp of |z*log2e - c| <= 2^-20 while the gap is below 32/log2e,
// i.e. below 7e-7 relative; c itself is carried exactly into the combine.
#include "csd_internal.h"

namespace csd {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRescaleGap = 20.0f;   // logit units; 20*log2e < 32 keeps the exponent's ulp at 2^-19 or finer
constexpr int kNoIter = 0x7fffffff;

// ---- wave-wide all-reduces: DPP inside a row of 16 lanes, ds_swizzle across rows, bpermute across halves
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

// ---- 16-byte chunk of logits -> fp32 values (bf16 widening is exact)
template <int DT> struct Chunk;
template <> struct Chunk<CSD_DTYPE_F32> {
    static constexpr int E = 4;
    static constexpr uint32_t kNegInfWord = 0xFF800000u;
    __device__ static __forceinline__ void unpack(const u32x4 &q, float (&x)[E]) {
        x[0] = __uint_as_float(q.x); x[1] = __uint_as_float(q.y);
        x[2] = __uint_as_float(q.z); x[3] = __uint_as_float(q.w);
    }
    __device__ static __forceinline__ float load_one(const char *row, int v) { return ((const float *)row)[v]; }
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
    __device__ static __forceinline__ float load_one(const char *row, int v) {
        return __uint_as_float((uint32_t)((const uint16_t *)row)[v] << 16);
    }
};

template <int E>
__device__ __forceinline__ float chunk_max(const float (&x)[E]) {
    float m = x[0];
#pragma unroll
    for (int j = 1; j < E; ++j) m = __builtin_fmaxf(m, x[j]);
    return m;
}

template <int DT>
__global__ __launch_bounds__(kStreamWaves *kWaveSize) void row_stream_kernel(const char *__restrict__ logits,
                                                                              int64_t row_pitch_bytes, int V, int nsplit,
                                                                              int chunks_per_split,
                                                                              RowPartial *__restrict__ partials) {
    using C = Chunk<DT>;
    constexpr int E = C::E;
    constexpr int W = kStreamWaves;
    constexpr int U = kStreamUnroll;

    const int row = blockIdx.x / nsplit;
    const int split = blockIdx.x - row * nsplit;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const char *rowp = logits + (int64_t)row * row_pitch_bytes;

    const int nfull = V / E;                       // whole 16-byte chunks of the row
    const int tail = V - nfull * E;                // logits in the ragged last chunk
    const int nchunks = nfull + (tail ? 1 : 0);
    const int c0 = split * chunks_per_split;       // this workgroup's chunk range [c0, c1)
    const int c1 = min(c0 + chunks_per_split, nchunks);
    const int cfull = min(c1, nfull);              // chunks below this are loaded whole
    const int ntiles = (cfull - c0) / kTileChunks; // tiles made of whole chunks only

    float rm = -INFINITY;      // running max of this lane
    int best_it = kNoIter;     // iteration that first reached rm
    float s[E];
#pragma unroll
    for (int j = 0; j < E; ++j) s[j] = 0.f;
    float c = 0.f;             // wave-uniform reference exponent (log2 units)
    float mth = -INFINITY;     // rescale when a lane maximum exceeds this

    // chunk visited by this lane at iteration it: c0 + (it*W + wave)*64 + lane
    const int lane_chunk0 = c0 + wave * kWaveSize + lane;

    auto rescale = [&]() {
        const float wm = wave_allreduce_f(rm, MaxF());
        const float cn = wm * kLog2e;
        const float sc = __builtin_amdgcn_exp2f(c - cn);
#pragma unroll
        for (int j = 0; j < E; ++j) s[j] = (s[j] == 0.f) ? 0.f : s[j] * sc;
        c = cn;
        mth = wm + kRescaleGap;
    };

    // ---- main loop: whole tiles, U independent 16-byte loads per lane
    const u32x4 *p = (const u32x4 *)rowp + lane_chunk0;
    for (int t = 0; t < ntiles; ++t) {
        u32x4 q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) q[u] = p[u * (W * kWaveSize)];
        p += U * (W * kWaveSize);

        float x[U][E];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            C::unpack(q[u], x[u]);
            const float cm = chunk_max<E>(x[u]);
            best_it = (cm > rm) ? (t * U + u) : best_it;
            rm = __builtin_fmaxf(rm, cm);
        }
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(rm > mth) != 0, 0)) rescale();
        const float nc = -c;
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int j = 0; j < E; ++j) s[j] += __builtin_amdgcn_exp2f(__builtin_fmaf(x[u][j], kLog2e, nc));
        }
    }

    // ---- remainder: one guarded chunk per lane per iteration (ragged chunk filled with -inf)
    for (int it = ntiles * U; c0 + it * (W * kWaveSize) < c1; ++it) {
        const int ch = lane_chunk0 + it * (W * kWaveSize);
        u32x4 q = {C::kNegInfWord, C::kNegInfWord, C::kNegInfWord, C::kNegInfWord};
        float x[E];
        if (ch < cfull) {
            q = ((const u32x4 *)rowp)[ch];
            C::unpack(q, x);
        } else {
            C::unpack(q, x);
            if (ch == nfull && ch < c1) {   // the ragged chunk: element loads, bounds-checked
#pragma unroll
                for (int j = 0; j < E; ++j)
                    if (j < tail) x[j] = C::load_one(rowp, nfull * E + j);
            }
        }
        const float cm = chunk_max<E>(x);
        best_it = (cm > rm) ? it : best_it;
        rm = __builtin_fmaxf(rm, cm);
        if (__builtin_amdgcn_ballot_w64(rm > mth) != 0) rescale();
        const float nc = -c;
#pragma unroll
        for (int j = 0; j < E; ++j) s[j] += __builtin_amdgcn_exp2f(__builtin_fmaf(x[j], kLog2e, nc));
    }

    // ---- wave result
    float sl = s[0];
#pragma unroll
    for (int j = 1; j < E; ++j) sl += s[j];
    const float ws = wave_allreduce_f(sl, AddF());
    const float wm = wave_allreduce_f(rm, MaxF());
    const int my_chunk = (best_it != kNoIter && rm == wm) ? (lane_chunk0 + best_it * (W * kWaveSize)) : kNoIter;
    const int bc = wave_allreduce_i(my_chunk, MinI());

    int idx = c0 * E;   // a segment without any finite value reports its first token
    if (bc != kNoIter) {
        // first element of the winning chunk equal to the maximum (float compare: -0 == +0)
        const int v = bc * E + lane;
        const bool hit = (lane < E) && (v < V) && (C::load_one(rowp, (lane < E && v < V) ? v : 0) == wm);
        const uint64_t mask = __builtin_amdgcn_ballot_w64(hit);
        idx = bc * E + (mask ? (int)__builtin_ctzll(mask) : 0);
    }
    if (lane == 0) {
        RowPartial out;
        out.m = wm;
        out.cref = c;
        out.s = ws;
        out.idx = idx;
        partials[((int64_t)row * nsplit + split) * W + wave] = out;
    }
}

}  // namespace

StreamPlan make_stream_plan(int B, int k, int V, int dtype) {
    StreamPlan p;
    p.rows = B * (k + 1);
    p.elems_per_chunk = (dtype == CSD_DTYPE_F32) ? 4 : 8;
    p.nchunks = (V + p.elems_per_chunk - 1) / p.elems_per_chunk;
    const int tiles = (p.nchunks + kTileChunks - 1) / kTileChunks;       // tiles per row, last one partial
    int want = p.rows > 0 ? (kTargetBlocks + p.rows - 1) / p.rows : 1;   // segments per row to fill the chip
    if (want < 1) want = 1;
    if (want > tiles) want = tiles;
    const int tiles_per_split = (tiles + want - 1) / want;
    p.chunks_per_split = tiles_per_split * kTileChunks;
    p.nsplit = (p.nchunks + p.chunks_per_split - 1) / p.chunks_per_split;   // every segment is non-empty
    p.partials_per_row = p.nsplit * kStreamWaves;
    return p;
}

hipError_t launch_row_stream(const void *logits, int dtype, int64_t row_stride, int V, const StreamPlan &plan,
                             RowPartial *partials, hipStream_t stream) {
    if (plan.rows == 0) return hipSuccess;
    const dim3 grid((unsigned)(plan.rows * plan.nsplit));
    const dim3 block(kStreamWaves * kWaveSize);
    if (dtype == CSD_DTYPE_F32) {
        hipLaunchKernelGGL(row_stream_kernel<CSD_DTYPE_F32>, grid, block, 0, stream, (const char *)logits, row_stride * 4, V,
                           plan.nsplit, plan.chunks_per_split, partials);
    } else {
        hipLaunchKernelGGL(row_stream_kernel<CSD_DTYPE_BF16>, grid, block, 0, stream, (const char *)logits, row_stride * 2, V,
                           plan.nsplit, plan.chunks_per_split, partials);
    }
    return hipGetLastError();
}

}  // namespace csd
