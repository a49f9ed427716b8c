// Eq. 1 of the paper: V_trim = V[Top-K(c, k)], W_trim = W[Top-K(c, k), :].
//
// select_topk_kernel: radix select of the k-th largest count (threshold T and the
//   number r of T-valued ids to keep; ties go to the lower id), then an
//   id-ordered compaction that emits the selected ids already ascending -- no sort.
//   One workgroup of 1024 threads: V is ~1e5 and the job is latency-bound.
// gather_rows_kernel: W_trim[j, :] = W[map[j], :], a pure copy at HBM speed.
#include "vt_build.h"
#include "vt_device.h"

namespace vt {

namespace {
constexpr int kSelWaves = kSelectThreads / kWave;   // 16
constexpr int kDigitBits = 8;
constexpr int kDigits = 1 << kDigitBits;
}  // namespace

__global__ void __launch_bounds__(kSelectThreads) select_topk_kernel(const long long *__restrict__ counts, int V,
                                                                     int k, int *__restrict__ map) {
    // 32 histogram copies indexed by lane: at most two lanes of one instruction share an address
    constexpr int kCopies = 32;
    __shared__ unsigned hist[kDigits * kCopies];
    __shared__ unsigned tot[kDigits];
    __shared__ unsigned long long s_wave[kSelWaves];
    __shared__ unsigned long long s_prefix;
    __shared__ int s_kk;
    __shared__ int s_gt[kSelWaves + 1], s_eq[kSelWaves + 1];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;

    // ---- largest count -> number of significant digits
    unsigned long long mx = 0;
    for (int v = tid; v < V; v += kSelectThreads) {
        const unsigned long long c = (unsigned long long)counts[v];
        mx = c > mx ? c : mx;
    }
    mx = wave_max_u64(mx);
    if (lane == 0) s_wave[w] = mx;
    __syncthreads();
    mx = 0;
    for (int q = 0; q < kSelWaves; ++q) mx = s_wave[q] > mx ? s_wave[q] : mx;
    const int nbits = mx == 0 ? 0 : 64 - __clzll((long long)mx);
    const int ndig = (nbits + kDigitBits - 1) / kDigitBits;
    if (tid == 0) {
        s_prefix = 0;
        s_kk = k;
    }
    __syncthreads();

    // ---- radix select, most significant digit first
    for (int p = ndig - 1; p >= 0; --p) {
        const int sh = p * kDigitBits;
        for (int b = tid; b < kDigits * kCopies; b += kSelectThreads) hist[b] = 0u;
        __syncthreads();
        const unsigned long long prefix = s_prefix;
        for (int v = tid; v < V; v += kSelectThreads) {
            const unsigned long long c = (unsigned long long)counts[v];
            const unsigned long long hi = (sh + kDigitBits >= 64) ? 0ull : (c >> (sh + kDigitBits));
            if (hi == prefix) atomicAdd(&hist[(unsigned)((c >> sh) & (kDigits - 1)) * kCopies + (lane & (kCopies - 1))], 1u);
        }
        __syncthreads();
        if (tid < kDigits) {
            unsigned s = 0;
            for (int q = 0; q < kCopies; ++q) s += hist[tid * kCopies + ((q + tid) & (kCopies - 1))];
            tot[tid] = s;
        }
        __syncthreads();
        if (tid == 0) {
            int kk = s_kk;
            unsigned cum = 0;
            int dg = kDigits - 1;
            for (; dg > 0; --dg) {
                if (cum + tot[dg] >= (unsigned)kk) break;
                cum += tot[dg];
            }
            s_kk = kk - (int)cum;
            s_prefix = (prefix << kDigitBits) | (unsigned)dg;
        }
        __syncthreads();
    }
    const unsigned long long T = s_prefix;   // the k-th largest count
    const int r = s_kk;                      // how many ids with count == T are kept (lowest ids)

    // ---- id-ordered compaction; wave w owns a contiguous id range
    const int span = ((V + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
    const int v0 = w * span, v1 = min(V, v0 + span);
    int ngt = 0, neq = 0;
    for (int v = v0 + lane; v < v0 + span; v += kWave) {
        const bool in = v < v1;
        const unsigned long long c = in ? (unsigned long long)counts[v] : 0ull;
        ngt += __popcll(__ballot(in && c > T));
        neq += __popcll(__ballot(in && c == T));
    }
    if (lane == 0) {
        s_gt[w + 1] = ngt;
        s_eq[w + 1] = neq;
    }
    __syncthreads();
    if (tid == 0) {
        s_gt[0] = 0;
        s_eq[0] = 0;
        for (int q = 1; q <= kSelWaves; ++q) {
            s_gt[q] += s_gt[q - 1];
            s_eq[q] += s_eq[q - 1];
        }
    }
    __syncthreads();
    int gbase = s_gt[w], ebase = s_eq[w];
    const unsigned long long lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    for (int v = v0 + lane; v < v0 + span; v += kWave) {
        const bool in = v < v1;
        const unsigned long long c = in ? (unsigned long long)counts[v] : 0ull;
        const bool gt = in && c > T, eq = in && c == T;
        const unsigned long long bg = __ballot(gt), be = __ballot(eq);
        const int gt_before = gbase + __popcll(bg & lt_mask);
        const int eq_before = ebase + __popcll(be & lt_mask);
        if (gt || (eq && eq_before < r)) map[gt_before + min(eq_before, r)] = v;
        gbase += __popcll(bg);
        ebase += __popcll(be);
    }
}

void launch_select_topk(const long long *counts, int V, int k, int *map, hipStream_t st) {
    hipLaunchKernelGGL(select_topk_kernel, dim3(1), dim3(kSelectThreads), 0, st, counts, V, k, map);
}

// One wave copies one row at a time with 16-byte lanes; rows are independent.
__global__ void __launch_bounds__(256) gather_rows_kernel(const char *__restrict__ W, size_t row_bytes,
                                                          const int *__restrict__ map, int k,
                                                          char *__restrict__ W_trim) {
    const int lane = lane_id();
    const int wave = (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    const int nwaves = (int)((gridDim.x * blockDim.x) >> 6);
    const size_t nvec = row_bytes >> 4;
    for (int j = wave; j < k; j += nwaves) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(W + (size_t)map[j] * row_bytes);
        u32x4 *dst = reinterpret_cast<u32x4 *>(W_trim + (size_t)j * row_bytes);
        size_t c = lane;
        for (; c + 3 * kWave < nvec; c += 4 * kWave) {
            const u32x4 a0 = __builtin_nontemporal_load(src + c);
            const u32x4 a1 = __builtin_nontemporal_load(src + c + kWave);
            const u32x4 a2 = __builtin_nontemporal_load(src + c + 2 * kWave);
            const u32x4 a3 = __builtin_nontemporal_load(src + c + 3 * kWave);
            __builtin_nontemporal_store(a0, dst + c);
            __builtin_nontemporal_store(a1, dst + c + kWave);
            __builtin_nontemporal_store(a2, dst + c + 2 * kWave);
            __builtin_nontemporal_store(a3, dst + c + 3 * kWave);
        }
        for (; c < nvec; c += kWave) __builtin_nontemporal_store(__builtin_nontemporal_load(src + c), dst + c);
    }
}

void launch_gather_rows(const void *W, size_t row_bytes, const int *map, int k, void *W_trim, hipStream_t st) {
    int blocks = (k + 3) / 4;          // 4 waves per workgroup
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const char *>(W), row_bytes,
                       map, k, static_cast<char *>(W_trim));
}

}  // namespace vt
