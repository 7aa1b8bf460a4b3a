// Internal declarations shared by the kernels and the C ABI (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "csd.h"

namespace csd {

// One wave's result for one segment of a logits row.
//   m    : maximum of the segment (-inf when the segment holds no finite value)
//   cref : reference exponent, in log2 units, that `s` is scaled by
//   s    : sum over the segment of 2^(z * log2e - cref)
//   idx  : lowest token id in the segment whose logit equals m
struct __attribute__((aligned(16))) RowPartial {
    float m;
    float cref;
    float s;
    int32_t idx;
};

constexpr int kWaveSize = 64;
constexpr int kStreamWaves = 4;              // waves per row-stream workgroup
constexpr int kStreamUnroll = 4;             // 16-byte loads in flight per lane
constexpr int kTileChunks = kStreamWaves * kWaveSize * kStreamUnroll;   // 16-byte chunks per workgroup iteration
constexpr int kTargetBlocks = 2048;          // row-stream grid size aimed at (8 per CU on 256 CUs)

// Launch plan of the row-stream kernel; a pure function of the shape so that the
// workspace size query and the launch agree.
struct StreamPlan {
    int rows;              // B * (k + 1)
    int elems_per_chunk;   // 4 (fp32) or 8 (bf16) logits per 16-byte chunk
    int nchunks;           // chunks per row, the ragged last one included
    int nsplit;            // segments per row
    int chunks_per_split;  // multiple of kTileChunks
    int partials_per_row;  // nsplit * kStreamWaves
};

StreamPlan make_stream_plan(int B, int k, int V, int dtype);

struct WorkspaceLayout {
    size_t partials_off, partials_bytes;
    size_t log_off, log_bytes;
    size_t total;
};

WorkspaceLayout make_workspace_layout(const StreamPlan &p, int B, int k);

// kernel launchers (enqueue only; return hipGetLastError())
hipError_t launch_row_stream(const void *logits, int dtype, int64_t row_stride, int V, const StreamPlan &plan,
                             RowPartial *partials, hipStream_t stream);

struct EpilogueArgs {
    const void *logits;
    int dtype;
    int64_t row_stride;
    const int32_t *draft;
    int B, k, V;
    float tau;
    uint32_t lambda;
    const uint64_t *ocm;
    uint64_t capacity;
    const RowPartial *partials;
    int partials_per_row;
    int32_t *accept_len;
    int32_t *next_token;
    int32_t *argmax;
    float *row_max;
    float *row_sumexp;
    float *ratio;
    float *p_draft;
    uint8_t *pos_flags;
    uint64_t *rej_log;      // user log or workspace log, may be NULL when nothing needs it
    uint32_t *status;
};

hipError_t launch_epilogue(const EpilogueArgs &a, hipStream_t stream);
hipError_t launch_ocm_update(uint64_t *ocm, uint64_t capacity, const uint64_t *keys, const uint32_t *weights, uint64_t n,
                             uint32_t *status, hipStream_t stream);
hipError_t launch_ocm_reset(uint64_t *ocm, uint64_t capacity, hipStream_t stream);
hipError_t launch_ocm_lookup(const uint64_t *ocm, uint64_t capacity, const uint64_t *keys, uint32_t *counts, uint64_t n,
                             hipStream_t stream);

}  // namespace csd
