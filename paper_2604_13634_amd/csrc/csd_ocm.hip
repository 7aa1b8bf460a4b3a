// Online Correction Memory maintenance kernels: bulk update (UpdateMemory as a separate call, and the
// load of a calibrated prior), reset, lookup.
#include "csd_device.h"

namespace csd {
namespace {

// Each workgroup takes kApplyBatch entries: merges duplicate keys in LDS, then issues one compare-and-swap
// chain per distinct key, so a skewed stream does not serialise on a handful of global slots.
__global__ __launch_bounds__(kApplyThreads) void ocm_update_kernel(uint64_t *ocm, uint64_t capacity,
                                                                   const uint64_t *__restrict__ keys,
                                                                   const uint32_t *__restrict__ weights, uint64_t n,
                                                                   uint32_t *status) {
    __shared__ ApplyLds lds;
    auto fetch = [&](uint64_t e, uint64_t &key, uint32_t &w) {
        key = keys[e] & CSD_OCM_KEY_MASK;
        w = weights ? weights[e] : 1u;
        if (w > CSD_OCM_COUNT_MAX) w = CSD_OCM_COUNT_MAX;
    };
    block_apply_batch(ocm, capacity, status, lds, fetch, (uint64_t)blockIdx.x * kApplyBatch, n);
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

}  // namespace

hipError_t launch_ocm_update(uint64_t *ocm, uint64_t capacity, const uint64_t *keys, const uint32_t *weights, uint64_t n,
                             uint32_t *status, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + kApplyBatch - 1) / kApplyBatch;
    hipLaunchKernelGGL(ocm_update_kernel, dim3((unsigned)blocks), dim3(kApplyThreads), 0, stream, ocm, capacity, keys, weights, n,
                       status);
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
