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

// Measurement reference: a kernel that only reads `nvec` 16-byte vectors once, in the launch shape
// and load shape of the small-n draft step (256 workgroups of 8 waves, 1 KiB per wave load,
// streaming hint, 8 loads in flight per lane) and folds them into a word per lane.  Its duration is
// what this machine takes to merely stream the bytes the step has to stream.
__global__ void __launch_bounds__(512) stream_read_kernel(const u32x4 *__restrict__ p, size_t nvec,
                                                          unsigned *__restrict__ sink) {
    const size_t per_block = (nvec + gridDim.x - 1) / gridDim.x;
    const size_t b0 = (size_t)blockIdx.x * per_block;
    const size_t b1 = b0 + per_block < nvec ? b0 + per_block : nvec;
    unsigned acc = 0u;
    size_t i = b0 + threadIdx.x;
    for (; i + 7 * 512 < b1; i += 8 * 512) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + i + (size_t)u * 512);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < b1; i += 512) {
        const u32x4 v = __builtin_nontemporal_load(p + i);
        acc += v.x ^ v.y ^ v.z ^ v.w;
    }
    // the fold is stored only if it hits one particular value: enough to keep the loads alive, and no
    // store or atomic traffic is added to what is being timed
    if (acc == 0x9E3779B9u) *sink = acc;
}

void launch_stream_read(const void *p, size_t bytes, unsigned *sink, hipStream_t st) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(256), dim3(512), 0, st, static_cast<const u32x4 *>(p), bytes / 16,
                       sink);
}

// ---- row gather / scatter around a step over a subset of the hidden rows (several heads per call)
// staging[b, :] = h[rows.idx[b], :]   (row_vecs 16-byte vectors per row)
__global__ void __launch_bounds__(256) gather_h_rows_kernel(const u32x4 *__restrict__ h, u32x4 *__restrict__ staging,
                                                            int row_vecs, const RowList rows) {
    const int b = blockIdx.x;
    const u32x4 *src = h + (size_t)rows.idx[b] * row_vecs;
    u32x4 *dst = staging + (size_t)b * row_vecs;
    for (int v = threadIdx.x; v < row_vecs; v += 256) dst[v] = src[v];
}
// out_*[rows.idx[b], :] = staged results of row b
__global__ void __launch_bounds__(64) scatter_rows_kernel(const int *__restrict__ ids_s, const float *__restrict__ logp_s,
                                                          const float *__restrict__ lse_s, int m,
                                                          int *__restrict__ out_ids, float *__restrict__ out_logp,
                                                          float *__restrict__ out_lse, const RowList rows) {
    const int b = blockIdx.x;
    const size_t dst = (size_t)rows.idx[b] * m, src = (size_t)b * m;
    for (int r = threadIdx.x; r < m; r += 64) {
        out_ids[dst + r] = ids_s[src + r];
        out_logp[dst + r] = logp_s[src + r];
    }
    if (out_lse != nullptr && threadIdx.x == 0) out_lse[rows.idx[b]] = lse_s[b];
}

void launch_gather_h_rows(const void *h, void *staging, size_t row_bytes, const RowList &rows, hipStream_t st) {
    hipLaunchKernelGGL(gather_h_rows_kernel, dim3(rows.n), dim3(256), 0, st, static_cast<const u32x4 *>(h),
                       static_cast<u32x4 *>(staging), (int)(row_bytes / 16), rows);
}
void launch_scatter_rows(const int *ids_s, const float *logp_s, const float *lse_s, int m, int *out_ids,
                         float *out_logp, float *out_lse, const RowList &rows, hipStream_t st) {
    hipLaunchKernelGGL(scatter_rows_kernel, dim3(rows.n), dim3(64), 0, st, ids_s, logp_s, lse_s, m, out_ids, out_logp,
                       out_lse, rows);
}

}  // namespace vt
