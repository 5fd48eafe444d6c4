// Plain device-to-device copy of a known number of bytes.  It exists so that
// hardware counters (bytes fetched / written per dispatch) can be scaled by
// what the same counters read for a transfer whose size is known exactly.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/specee.h"

namespace specee {

__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4 *src, uint4 *dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace specee

extern "C" int specee_calib_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return SPECEE_EINVAL;
    if (bytes == 0) return SPECEE_OK;
    size_t n16 = bytes / 16;
    size_t wgs = (n16 + 255) / 256;
    if (wgs > 256 * 16) wgs = 256 * 16;
    hipLaunchKernelGGL(specee::calib_copy_kernel, dim3((unsigned)wgs), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n16);
    return hipGetLastError() == hipSuccess ? SPECEE_OK : SPECEE_EHIP;
}
