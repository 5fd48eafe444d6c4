// Device status word: conditions that only the device can see (a speculative id outside the vocabulary,
// a tree whose merged set exceeds its capacity) are reported in the outputs themselves -- NaN scores, the
// true size in M_out.  This kernel folds them into one int32 on the device, so that a caller reads one
// word after its synchronisation instead of scanning the outputs on the host.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/specee.h"

namespace specee {

__global__ __launch_bounds__(256) void status_kernel(const float *scores, size_t n_scores, const int32_t *M_out, int G,
                                                     int Mcap, int32_t *status) {
    __shared__ int any[2];
    if (threadIdx.x < 2) any[threadIdx.x] = 0;
    __syncthreads();
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    int bad = 0, over = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_scores; i += stride) {
        const float s = scores[i];
        bad |= s != s;
    }
    if (M_out)
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < (size_t)G; i += stride) over |= M_out[i] > Mcap;
    if (bad) any[0] = 1;   // benign race: all writers store 1
    if (over) any[1] = 1;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int bits = (any[0] ? SPECEE_STATUS_INVALID_ID : 0) | (any[1] ? SPECEE_STATUS_MERGE_OVERFLOW : 0);
        if (bits) atomicOr(status, bits);
    }
}

__global__ void status_clear_kernel(int32_t *status) {
    *status = 0;
}

}  // namespace specee

extern "C" int specee_status_word(const float *scores, size_t n_scores, const int32_t *M_out, int G, int Mcap,
                                  int32_t *status, void *stream) {
    if (!status || (n_scores > 0 && !scores) || G < 0 || (G > 0 && M_out && Mcap < 1)) return SPECEE_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(specee::status_clear_kernel, dim3(1), dim3(1), 0, st, status);
    const size_t work = n_scores > (size_t)G ? n_scores : (size_t)G;
    if (work > 0) {
        size_t wgs = (work + 255) / 256;
        if (wgs > 1024) wgs = 1024;
        hipLaunchKernelGGL(specee::status_kernel, dim3((unsigned)wgs), dim3(256), 0, st, scores, n_scores,
                           M_out ? M_out : nullptr, M_out ? G : 0, Mcap, status);
    }
    return hipGetLastError() == hipSuccess ? SPECEE_OK : SPECEE_EHIP;
}
