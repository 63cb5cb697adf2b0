// lsm_build_fences: fence-pointer index of a sorted run (paper section 2.2 names fence
// pointers as the structure that makes lookups efficient).  fence[i] = key of entry i*stride.
#include <hip/hip_runtime.h>

#include "lsm_common.h"

namespace lsm {

// Two lanes per fence, 16 bytes each: the 32-byte stores of a wave are contiguous.
__global__ void __launch_bounds__(256) fence_kernel(const lsm_entry_t* run, uint64_t n_fences, uint64_t stride, uint4* out) {
    uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t step = (uint64_t)gridDim.x * blockDim.x;
    for (; g < n_fences * 2; g += step) {
        uint64_t i = g >> 1;
        uint32_t half = (uint32_t)(g & 1);
        out[g] = reinterpret_cast<const uint4*>(run + i * stride)[half];
    }
}

}  // namespace lsm

extern "C" int lsm_build_fences(const lsm_run_t* run, uint32_t stride, uint8_t* fence_keys_out, void* stream) {
    if (run == nullptr) return LSM_ERR_NULL;
    if (stride == 0) return LSM_ERR_BAD_ARG;
    if (run->n == 0) return LSM_OK;
    if (run->entries == nullptr || fence_keys_out == nullptr) return LSM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(run->entries) & 63) != 0 || (reinterpret_cast<uintptr_t>(fence_keys_out) & 15) != 0)
        return LSM_ERR_BAD_ARG;
    uint64_t n_fences = (run->n + stride - 1) / stride;
    uint64_t blocks = (n_fences * 2 + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(lsm::fence_kernel, dim3((uint32_t)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), run->entries,
                       n_fences, (uint64_t)stride, reinterpret_cast<uint4*>(fence_keys_out));
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}
