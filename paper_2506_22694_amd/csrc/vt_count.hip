// Algorithm 1 (Count Token Frequencies): c[t] += 1 for every token id of the stream.
//
// The V counters do not fit one CU's LDS (V = 128256 -> 513 KB as uint32), so
// the vocabulary is cut into ranges of 32768 bins (128 KiB of LDS) and the id
// stream into chunks.  Workgroup (chunk, range) reads its chunk with 16-byte
// loads, counts the ids that fall into its range with LDS atomics (no global
// atomic ever sees the Zipf-hot ids), and writes its private histogram to
// scratch.  A second kernel sums the chunk histograms into the caller's int64
// counters.  Ids outside [0, V) are skipped and tallied.
#include "vt_build.h"
#include "vt_device.h"

namespace vt {

int hist_num_ranges(int V) { return (V + kHistBinsPerBlock - 1) / kHistBinsPerBlock; }

int hist_num_chunks(int64_t n_ids) {
    // at least 128K ids per chunk so that zeroing and flushing 128 KiB of LDS pays off
    int64_t c = (n_ids + (1 << 17) - 1) >> 17;
    if (c < 1) c = 1;
    if (c > kHistMaxChunks) c = kHistMaxChunks;
    return (int)c;
}

// `head` ids (fewer than one 16-byte vector) precede the first 16-byte aligned id.
template <bool IDS64>
__global__ void __launch_bounds__(kHistThreads) hist_partial_kernel(const void *__restrict__ ids_v, long long n_ids,
                                                                    int head, int V, int nchunks,
                                                                    unsigned *__restrict__ partial,
                                                                    unsigned long long *__restrict__ n_invalid) {
    extern __shared__ __align__(16) unsigned bins[];
    const int chunk = blockIdx.x, range = blockIdx.y;
    const int lo = range * kHistBinsPerBlock;
    const int nb = min(kHistBinsPerBlock, V - lo);
    for (int b = threadIdx.x; b < nb; b += kHistThreads) bins[b] = 0u;
    __syncthreads();

    // chunk boundaries in units of 16-byte vectors (4 int32 or 2 int64), tail handled by the last chunk
    constexpr int IPV = IDS64 ? 2 : 4;
    constexpr int IDB = IDS64 ? 8 : 4;
    const long long nvec = (n_ids - head) / IPV;
    const long long v0 = nvec * chunk / nchunks, v1 = nvec * (chunk + 1) / nchunks;
    unsigned invalid = 0;
    auto tally = [&](long long t) {
        if (t < 0 || t >= (long long)V) {
            invalid += 1u;
        } else {
            const unsigned b = (unsigned)((int)t - lo);
            if (b < (unsigned)nb) atomicAdd(&bins[b], 1u);
        }
    };
    const u32x4 *vp = reinterpret_cast<const u32x4 *>(static_cast<const char *>(ids_v) + (size_t)head * IDB);
    auto tally_vec = [&](const u32x4 q) {
        if constexpr (IDS64) {
            tally((long long)(((unsigned long long)q.y << 32) | q.x));
            tally((long long)(((unsigned long long)q.w << 32) | q.z));
        } else {
            tally((long long)(int)q.x);
            tally((long long)(int)q.y);
            tally((long long)(int)q.z);
            tally((long long)(int)q.w);
        }
    };
    // kHistUnroll vectors per thread are requested before the first is counted: one 16-byte load per
    // thread in flight (16 KiB per CU) is far below what the memory latency needs.  Plain (cached) loads:
    // the workgroups of one chunk (one per range) are dispatched to the same XCD and read the same ids at
    // about the same time, so three of the four reads can hit its L2; a streaming hint would drop the
    // lines after the first use (10^7 ids: 41.2 -> 35.1 us)
    long long v = v0 + threadIdx.x;
    for (; v + (long long)(kHistUnroll - 1) * kHistThreads < v1; v += (long long)kHistUnroll * kHistThreads) {
        u32x4 q[kHistUnroll];
#pragma unroll
        for (int u = 0; u < kHistUnroll; ++u) q[u] = vp[v + (long long)u * kHistThreads];
#pragma unroll
        for (int u = 0; u < kHistUnroll; ++u) tally_vec(q[u]);
    }
    for (; v < v1; v += kHistThreads) tally_vec(vp[v]);
    if (chunk == 0 && (int)threadIdx.x < head) {   // scalar head
        if constexpr (IDS64) tally(static_cast<const long long *>(ids_v)[threadIdx.x]);
        else tally((long long)static_cast<const int *>(ids_v)[threadIdx.x]);
    }
    if (chunk == nchunks - 1) {   // scalar tail (< IPV ids)
        const long long i = head + nvec * IPV + threadIdx.x;
        if (i < n_ids) {
            if constexpr (IDS64) tally(static_cast<const long long *>(ids_v)[i]);
            else tally((long long)static_cast<const int *>(ids_v)[i]);
        }
    }
    __syncthreads();
    unsigned *dst = partial + (size_t)chunk * V + lo;
    for (int b = threadIdx.x; b < nb; b += kHistThreads) dst[b] = bins[b];
    // every range-workgroup of a chunk sees the same invalid ids: only range 0 reports them
    if (n_invalid != nullptr && range == 0) {
        const int tot = wave_sum_i32((int)invalid);
        if (lane_id() == 0 && tot != 0) atomicAdd(n_invalid, (unsigned long long)tot);
    }
}

__global__ void __launch_bounds__(256) hist_reduce_kernel(const unsigned *__restrict__ partial, int nchunks, int V,
                                                          long long *__restrict__ counts) {
    const int v = blockIdx.x * 256 + threadIdx.x;
    if (v >= V) return;
    long long s = 0;
    int c = 0;
    for (; c + 8 <= nchunks; c += 8) {
        unsigned t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = partial[(size_t)(c + u) * V + v];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += (long long)t[u];
    }
    for (; c < nchunks; ++c) s += (long long)partial[(size_t)c * V + v];
    counts[v] += s;
}

hipError_t launch_count_tokens(const void *ids, bool ids64, int64_t n_ids, int V, long long *counts,
                         unsigned long long *n_invalid, unsigned *partial, hipStream_t st) {
    const int nchunks = hist_num_chunks(n_ids);
    const int nranges = hist_num_ranges(V);
    const size_t lds = (size_t)kHistBinsPerBlock * sizeof(unsigned);
    static bool attr_set[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(hist_partial_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(hist_partial_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    dim3 grid(nchunks, nranges);
    // ids before the first 16-byte boundary are counted one by one
    const int idb = ids64 ? 8 : 4;
    const uintptr_t mis = reinterpret_cast<uintptr_t>(ids) & 15u;
    long long head = mis ? (long long)((16 - mis) / idb) : 0;
    if (head > n_ids) head = n_ids;
    if (ids64)
        hipLaunchKernelGGL(hist_partial_kernel<true>, grid, dim3(kHistThreads), lds, st, ids, (long long)n_ids,
                           (int)head, V, nchunks, partial, n_invalid);
    else
        hipLaunchKernelGGL(hist_partial_kernel<false>, grid, dim3(kHistThreads), lds, st, ids, (long long)n_ids,
                           (int)head, V, nchunks, partial, n_invalid);
    hipLaunchKernelGGL(hist_reduce_kernel, dim3((V + 255) / 256), dim3(256), 0, st, partial, nchunks, V, counts);
    return hipGetLastError();
}

}  // namespace vt
