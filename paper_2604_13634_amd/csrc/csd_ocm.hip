// Online Correction Memory maintenance kernels: bulk update (UpdateMemory as a separate call, and the
// load of a calibrated prior), reset, lookup.
#include "csd_device.h"

namespace csd {
namespace {

// A fixed grid of workgroups walks the list, kApplyBatch entries at a time per workgroup: duplicate keys are
// merged in LDS across everything a workgroup sees, then one compare-and-swap chain per distinct key goes
// to the table, so a skewed stream does not serialise on a handful of global slots.
constexpr unsigned kUpdateGrid = 1024;
__global__ __launch_bounds__(kApplyThreads) void ocm_update_kernel(uint64_t *ocm, uint64_t capacity,
                                                                   const uint64_t *__restrict__ keys,
                                                                   const uint32_t *__restrict__ weights, uint64_t n,
                                                                   const uint64_t *__restrict__ n_dev, uint32_t *status) {
    __shared__ ApplyLds lds;
    if (n_dev != nullptr) {                         // the list's length as the device knows it, never beyond the arrays
        const uint64_t nd = *n_dev;
        n = nd < n ? nd : n;
    }
    auto fetch = [&](uint64_t e, uint64_t &key, uint32_t &w) {
        key = keys[e] & CSD_OCM_KEY_MASK;
        w = weights ? weights[e] : 1u;
        if (w > CSD_OCM_COUNT_MAX) w = CSD_OCM_COUNT_MAX;
    };
    block_apply_list(ocm, capacity, status, lds, fetch, blockIdx.x, gridDim.x, n);
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

// every pair of src goes into dst with its count; keys of one table are distinct, so no merging first
__global__ void ocm_merge_kernel(uint64_t *dst, uint64_t dst_capacity, const uint64_t *__restrict__ src,
                                 uint64_t src_capacity, uint32_t *status) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < src_capacity; i += stride) {
        const uint64_t s = src[i];
        const uint64_t key = slot_key(s);
        const uint32_t w = slot_count(s);
        if (key == CSD_OCM_EMPTY || w == 0) continue;
        if (!ocm_add(dst, dst_capacity, key, w) && status) atomicAdd(&status[CSD_STATUS_DROPPED], w);
    }
}

__global__ void zero_u64_kernel(unsigned long long *p) { *p = 0; }

// compaction: a wave reads kExportLoads x 64 consecutive slots, reserves room for all their occupied ones with
// ONE atomic (waves adding to the one counter are what this kernel waits for), then writes them out
constexpr int kExportLoads = 16;
__global__ void ocm_export_kernel(const uint64_t *__restrict__ ocm, uint64_t capacity, uint64_t *__restrict__ keys_out,
                                  uint32_t *__restrict__ counts_out, uint64_t max_entries, unsigned long long *n_out) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    const uint64_t wave_id = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWaveSize;
    const uint64_t waves = (uint64_t)gridDim.x * blockDim.x / kWaveSize;
    const uint64_t span = (uint64_t)kExportLoads * kWaveSize;
    for (uint64_t base = wave_id * span; base < capacity; base += waves * span) {     // wave-uniform bounds
        uint64_t s[kExportLoads];
        unsigned int total = 0;
#pragma unroll
        for (int u = 0; u < kExportLoads; ++u) {
            const uint64_t i = base + (uint64_t)u * kWaveSize + lane;
            s[u] = (i < capacity) ? ocm[i] : CSD_OCM_EMPTY;
            total += (unsigned int)__builtin_popcountll(__builtin_amdgcn_ballot_w64(slot_key(s[u]) != CSD_OCM_EMPTY));
        }
        if (total == 0) continue;
        unsigned long long start = 0;
        if (lane == 0) start = atomicAdd(n_out, (unsigned long long)total);
        start = ((unsigned long long)__builtin_amdgcn_readfirstlane((int)(start >> 32)) << 32) |
                (unsigned int)__builtin_amdgcn_readfirstlane((int)(start & 0xFFFFFFFFull));
#pragma unroll
        for (int u = 0; u < kExportLoads; ++u) {
            const bool used = slot_key(s[u]) != CSD_OCM_EMPTY;
            const uint64_t mask = __builtin_amdgcn_ballot_w64(used);
            if (used) {
                const uint64_t pos = start + (uint64_t)__builtin_popcountll(mask & ((1ull << lane) - 1ull));
                if (pos < max_entries) {
                    keys_out[pos] = slot_key(s[u]);
                    counts_out[pos] = slot_count(s[u]);
                }
            }
            start += (unsigned long long)__builtin_popcountll(mask);
        }
    }
}

}  // namespace

hipError_t launch_ocm_merge(uint64_t *dst, uint64_t dst_capacity, const uint64_t *src, uint64_t src_capacity,
                            uint32_t *status, hipStream_t stream) {
    uint64_t blocks = (src_capacity + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(ocm_merge_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, dst, dst_capacity, src, src_capacity,
                       status);
    return hipGetLastError();
}

hipError_t launch_ocm_export(const uint64_t *ocm, uint64_t capacity, uint64_t *keys_out, uint32_t *counts_out,
                             uint64_t max_entries, uint64_t *n_out, hipStream_t stream) {
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, stream, (unsigned long long *)n_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    uint64_t blocks = (capacity + 256 * kExportLoads - 1) / (256 * kExportLoads);   // a workgroup of 4 waves covers 4096 slots a round
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(ocm_export_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, ocm, capacity, keys_out, counts_out,
                       max_entries, (unsigned long long *)n_out);
    return hipGetLastError();
}

hipError_t launch_ocm_update(uint64_t *ocm, uint64_t capacity, const uint64_t *keys, const uint32_t *weights, uint64_t n,
                             const uint64_t *n_dev, uint32_t *status, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    uint64_t blocks = (n + kApplyBatch - 1) / kApplyBatch;
    if (blocks > kUpdateGrid) blocks = kUpdateGrid;
    hipLaunchKernelGGL(ocm_update_kernel, dim3((unsigned)blocks), dim3(kApplyThreads), 0, stream, ocm, capacity, keys, weights, n,
                       n_dev, status);
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
