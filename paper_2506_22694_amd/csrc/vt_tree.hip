// Draft-tree growth downstream of the draft head (Sec. 4.1, "Draft Tree": depth 3, top-K 8, at
// most 32 tokens; Sec. 4.2 ablates deeper trees with 60 tokens): per level, candidate (i, j) =
// child j of frontier node i scores cum[i] + logp[i][j] and the K best become the next frontier;
// at the end the T best of all drafted nodes are kept in node order.
//
// Both are "the K largest of N keys, ties to the lower index", N = n * m being 64 for the
// paper's tree and a few hundred for the rerank.  One workgroup:
//   N <= 1024: every candidate finds its rank by counting the keys above its own (the keys sit in
//              LDS and every lane of a wave reads the same one: a broadcast, no bank conflicts);
//              1024 / N2 threads share one candidate's scan.  No sort, two barriers.
//   N  > 1024: bitonic sort of the 64-bit keys in LDS.
// key = orderable(score) << 32 | ~index, as in the draft step, so keys are distinct and "larger
// key" is "better score, then lower index".
#include "vt_tree.h"
#include "vt_device.h"
#include "vt_launch.h"
#include "vt_tree_dev.h"

namespace vt {

namespace {

__global__ void __launch_bounds__(kTreeThreads) tree_count_kernel(const TreeArgs a, int N2) {
    __shared__ unsigned long long keys[kTreeCountMaxN];
    __shared__ unsigned cnt[kTreeCountMaxN];
    __shared__ int wave_tot[kTreeThreads / kWave];
    tree_select_by_count<kTreeThreads, false>(a, N2, keys, cnt, wave_tot);
}

// descending bitonic sort of n2 (a power of two) keys in LDS by all threads of the workgroup
__device__ void bitonic_sort_desc(unsigned long long *keys, int n2) {
    for (int size = 2; size <= n2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = threadIdx.x; t < (n2 >> 1); t += blockDim.x) {
                const int lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                const int hi = lo | stride;
                const bool desc = (lo & size) == 0;
                const unsigned long long x = keys[lo], y = keys[hi];
                if ((x < y) == desc) {
                    keys[lo] = y;
                    keys[hi] = x;
                }
            }
        }
    }
    __syncthreads();
}

__global__ void __launch_bounds__(kTreeThreads) tree_sort_kernel(const TreeArgs a, int N2, int K2) {
    extern __shared__ __align__(16) unsigned long long skeys[];
    for (int c = threadIdx.x; c < N2; c += kTreeThreads) skeys[c] = tree_key<false>(a, c);
    bitonic_sort_desc(skeys, N2);
    if (!a.index_order) {
        for (int r = threadIdx.x; r < a.K; r += kTreeThreads)
            tree_emit(a, r, skeys[r], tree_token<false>(a, key_id(skeys[r])));
        return;
    }
    // the K winners, re-keyed by index alone (~index descending = index ascending), sorted again
    unsigned long long mine[kTreeMaxKeepSorted / kTreeThreads];
#pragma unroll
    for (int q = 0; q < kTreeMaxKeepSorted / kTreeThreads; ++q) {
        const int r = threadIdx.x + q * kTreeThreads;
        mine[q] = r < a.K ? skeys[r] : kNoKey;
    }
    __syncthreads();
    unsigned long long *byidx = skeys + N2 / 2;    // N2 >= 2048 > 2 * K2: the halves do not overlap
#pragma unroll
    for (int q = 0; q < kTreeMaxKeepSorted / kTreeThreads; ++q) {
        const int r = threadIdx.x + q * kTreeThreads;
        // sort key = (~index) << 32 | orderable score: distinct, ordered by index alone
        if (r < K2) byidx[r] = r < a.K ? ((mine[q] << 32) | (mine[q] >> 32)) : kNoKey;
    }
    bitonic_sort_desc(byidx, K2);
    for (int r = threadIdx.x; r < a.K; r += kTreeThreads) {
        const unsigned long long s = byidx[r];
        const unsigned long long key = (s << 32) | (s >> 32);
        tree_emit(a, r, key, tree_token<false>(a, key_id(key)));
    }
}

int pow2_at_least(int x, int lo) {
    int p = lo;
    while (p < x) p <<= 1;
    return p;
}

}  // namespace

hipError_t launch_tree_select(const TreeArgs &a, hipStream_t st) {
    if (a.N <= kTreeCountMaxN) {
        const int N2 = pow2_at_least(a.N, kWave);
        hipLaunchKernelGGL(tree_count_kernel, dim3(1), dim3(kTreeThreads), 0, st, a, N2);
        return hipGetLastError();
    }
    const int N2 = pow2_at_least(a.N, 2 * kTreeCountMaxN);
    const int K2 = pow2_at_least(a.K, 2);
    const size_t lds = (size_t)N2 * sizeof(unsigned long long);
    static LdsLimitOnce lds_limit;
    hipError_t e = allow_dynamic_lds(lds_limit, {reinterpret_cast<const void *>(tree_sort_kernel)},
                                     (int)(kTreeMaxN * sizeof(unsigned long long)));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(tree_sort_kernel, dim3(1), dim3(kTreeThreads), lds, st, a, N2, K2);
    return hipGetLastError();
}

}  // namespace vt
