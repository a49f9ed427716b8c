// Small helper kernels of the draft step.
#include "vt_device.h"
#include "vt_step.h"

namespace vt {

// out_logp_full holds raw logits after the main kernel; subtract the row's lse.
__global__ void __launch_bounds__(256) sub_lse_kernel(float *__restrict__ logp_full, const float *__restrict__ lse,
                                                      int n, int k) {
    const int i = blockIdx.y;
    const float l = lse[i];
    float *row = logp_full + (size_t)i * k;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < k; j += gridDim.x * blockDim.x) row[j] -= l;
}

void launch_sub_lse(float *logp_full, const float *lse, int n, int k, hipStream_t st) {
    int gx = (k + 255) / 256;
    if (gx > 1024) gx = 1024;
    hipLaunchKernelGGL(sub_lse_kernel, dim3(gx, n), dim3(256), 0, st, logp_full, lse, n, k);
}

__global__ void __launch_bounds__(64) ws_clear_kernel(unsigned *p, int nwords) {
    for (int i = threadIdx.x; i < nwords; i += 64) p[i] = 0u;
}

void launch_ws_clear(unsigned *p, int nwords, hipStream_t st) {
    hipLaunchKernelGGL(ws_clear_kernel, dim3(1), dim3(64), 0, st, p, nwords);
}

}  // namespace vt
