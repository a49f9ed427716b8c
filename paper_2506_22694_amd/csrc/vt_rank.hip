// Frequency-rank order and the alternative choices of k (Sec. 3.2: besides a fixed k, Top-P over
// the counts or a minimum-frequency threshold select the trimmed vocabulary).
//
// Rank order = all V ids sorted by (count descending, id ascending), the order in which
// Top-K(c, k) takes ids; every prefix is the selection for a smaller k.
//
// rsort_*: stable LSD radix sort of the (count, id) pairs over the whole device, 8 bits per pass.
//   The ids start ascending and every pass is stable, so equal counts stay in ascending-id order.
//   One workgroup per 1024 consecutive elements; a wave takes 64 consecutive elements, lanes with
//   equal digits find each other with nine ballots and rank themselves by population count, so
//   "earlier in the input" is (workgroup, wave, lane) order and no per-thread histogram is needed.
//     rsort_init     keys/ids from the counts, and the digit totals of all eight byte positions
//     rsort_hist     per-workgroup digit histogram of one pass
//     rsort_scatter  every workgroup derives its own output offsets from the histogram table
//                    (sum over earlier digits and over earlier workgroups), then scatters
//   A pass whose digit is the same for every key moves nothing and is skipped: each kernel
//   derives that, and which buffer currently holds the data, from the digit totals alone, so the
//   host enqueues a fixed sequence without reading anything back.  With 10^7 calibration tokens
//   three of the eight passes do work.
// choose_*: prefix sums over the sorted counts (per-workgroup sums, then every workgroup places itself in the
//   running mass); the smallest prefix whose mass reaches ceil(P * total), or the number of counts >= f_min.
#include "vt_build.h"
#include "vt_device.h"

namespace vt {

namespace {

inline size_t round256(size_t x) { return (x + 255) / 256 * 256; }

constexpr int kSortWaves = kRankSortThreads / kWave;   // 16
constexpr int kDigits = 256;
constexpr int kPasses = 8;

struct SortBufs {
    unsigned long long *keys[2];
    int *ids[2];
    unsigned *gtot;      // [kPasses][kDigits] digit totals over all elements
    unsigned *hist;      // [kDigits][nblk] per-workgroup digit counts of the current pass, descending digit first
};

// lanes of the wave whose `dgt` (0..256, 256 = not an element) equals this lane's
__device__ __forceinline__ unsigned long long match_digit9(int dgt) {
    unsigned long long m = ~0ull;
#pragma unroll
    for (int b = 0; b < 9; ++b) {
        const bool bit = (dgt >> b) & 1;
        const unsigned long long B = __ballot(bit);
        m &= bit ? B : ~B;
    }
    return m;
}
__device__ __forceinline__ int lanes_below(unsigned long long m) {
    return (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
}

// A pass is idle iff one digit bin holds all n elements.  Every wave of every kernel evaluates this
// the same way from the digit totals (call with all 64 lanes active).
__device__ __forceinline__ bool pass_active(const unsigned *__restrict__ gtot, int p, int n) {
    bool idle = false;
    for (int d = (int)threadIdx.x & 63; d < kDigits; d += kWave) idle |= gtot[p * kDigits + d] == (unsigned)n;
    return __ballot(idle) == 0ull;
}
// Buffer (0 or 1) that holds the data before pass p: the parity of the active passes before it.
__device__ __forceinline__ int source_buffer(const unsigned *__restrict__ gtot, int p, int n) {
    int moved = 0;
    for (int q = 0; q < p; ++q) moved += pass_active(gtot, q, n) ? 1 : 0;
    return moved & 1;
}

// Every later kernel copies the digit totals (8 KiB) into LDS first: pass_active / source_buffer read them
// many times over.
template <int T>
__device__ __forceinline__ void stage_totals(const unsigned *__restrict__ gtot, unsigned *gs) {
    for (int i = threadIdx.x; i < kPasses * kDigits; i += T) gs[i] = gtot[i];
    __syncthreads();
}

__global__ void __launch_bounds__(256) rsort_zero_kernel(unsigned *gtot) {
    for (int i = threadIdx.x; i < kPasses * kDigits; i += 256) gtot[i] = 0u;
}

__global__ void __launch_bounds__(kRankSortThreads) rsort_init_kernel(const long long *__restrict__ counts, int n,
                                                                      SortBufs b) {
    __shared__ unsigned h[kPasses * kDigits];
    for (int i = threadIdx.x; i < kPasses * kDigits; i += kRankSortThreads) h[i] = 0u;
    __syncthreads();
    const int j = blockIdx.x * kRankSortThreads + threadIdx.x;
    if (j < n) {
        const unsigned long long c = (unsigned long long)counts[j];
        b.keys[0][j] = c;
        b.ids[0][j] = j;
    }
    // the upper bytes are the same in nearly every key (zero): when a whole wave agrees on a digit one lane
    // adds for all, instead of 64 LDS atomics queueing on one address
    {
        const unsigned long long c = j < n ? (unsigned long long)counts[j] : 0ull;
        const unsigned long long live = __ballot(j < n);
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int dg = (int)((c >> (8 * p)) & 255ull);
            const int first = __builtin_amdgcn_readfirstlane(dg);
            const unsigned long long same = __ballot(j < n && dg == first);
            if (same == live && live != 0ull) {
                if ((threadIdx.x & 63) == (unsigned)(__ffsll((long long)live) - 1))
                    atomicAdd(&h[p * kDigits + dg], (unsigned)__popcll(live));
            } else if (j < n) {
                atomicAdd(&h[p * kDigits + dg], 1u);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kPasses * kDigits; i += kRankSortThreads) {
        if (h[i] != 0u) atomicAdd(&b.gtot[i], h[i]);
    }
}

__global__ void __launch_bounds__(kRankSortThreads) rsort_hist_kernel(int n, int p, SortBufs b) {
    __shared__ unsigned h[kDigits];
    __shared__ unsigned gs[kPasses * kDigits];
    stage_totals<kRankSortThreads>(b.gtot, gs);
    if (!pass_active(gs, p, n)) return;
    const int src = source_buffer(gs, p, n);
    if (threadIdx.x < kDigits) h[threadIdx.x] = 0u;
    __syncthreads();
    const int j = blockIdx.x * kRankSortThreads + threadIdx.x;
    if (j < n) atomicAdd(&h[255 - (int)((b.keys[src][j] >> (8 * p)) & 255ull)], 1u);
    __syncthreads();
    if (threadIdx.x < kDigits) b.hist[threadIdx.x * gridDim.x + blockIdx.x] = h[threadIdx.x];
}

__global__ void __launch_bounds__(kRankSortThreads) rsort_scatter_kernel(int n, int p, SortBufs b) {
    __shared__ unsigned wcnt[kSortWaves * kDigits];   // [wave][digit]: elements of that digit in earlier waves
    __shared__ unsigned part[4 * kDigits];            // sums over a quarter of the earlier workgroups
    __shared__ unsigned offs[kDigits];                // first output slot of this workgroup's run of each digit
    __shared__ unsigned gs[kPasses * kDigits];
    stage_totals<kRankSortThreads>(b.gtot, gs);
    if (!pass_active(gs, p, n)) return;
    const int src = source_buffer(gs, p, n);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nblk = gridDim.x, blk = blockIdx.x;

    for (int i = tid; i < kSortWaves * kDigits; i += kRankSortThreads) wcnt[i] = 0u;
    // this workgroup's offsets: (elements with an earlier digit anywhere) + (same digit, earlier workgroups)
    {
        const int d = tid >> 2, q = tid & 3;
        unsigned before = 0;
        const int b0 = nblk * q / 4, b1 = nblk * (q + 1) / 4;
        const int b1c = b1 < blk ? b1 : blk;
        const unsigned *row = b.hist + (size_t)d * nblk;
        int x = b0;
        for (; x + 8 <= b1c; x += 8) {          // eight independent loads at a time
            unsigned t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = row[x + u];
#pragma unroll
            for (int u = 0; u < 8; ++u) before += t[u];
        }
        for (; x < b1c; ++x) before += row[x];
        part[q * kDigits + d] = before;
    }
    unsigned tot = 0, inc = 0;
    if (tid < kDigits) {
        tot = gs[p * kDigits + (255 - tid)];          // digit totals in descending-digit order
        inc = tot;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {         // inclusive scan inside each of the four waves
            const unsigned t = __shfl_up(inc, o);
            if (lane >= o) inc += t;
        }
        offs[tid] = inc;
    }
    __syncthreads();
    unsigned my_off = 0;
    if (tid < kDigits) {
        unsigned carry = 0;
        for (int ww = 0; ww < w; ++ww) carry += offs[ww * kWave + kWave - 1];
        my_off = carry + inc - tot + part[tid] + part[kDigits + tid] + part[2 * kDigits + tid] + part[3 * kDigits + tid];
    }
    __syncthreads();
    if (tid < kDigits) offs[tid] = my_off;

    // ---- ranks inside the workgroup
    const int j = blk * kRankSortThreads + tid;
    const bool in = j < n;
    const unsigned long long key = in ? b.keys[src][j] : 0ull;
    const int idv = in ? b.ids[src][j] : 0;
    const int dgt = in ? 255 - (int)((key >> (8 * p)) & 255ull) : 256;
    const unsigned long long m = match_digit9(dgt);
    const int below = lanes_below(m);
    if (in && below == 0) wcnt[w * kDigits + dgt] = (unsigned)__popcll(m);
    __syncthreads();
    if (tid < kDigits) {
        unsigned run = 0;
        for (int ww = 0; ww < kSortWaves; ++ww) {
            const unsigned c = wcnt[ww * kDigits + tid];
            wcnt[ww * kDigits + tid] = run;
            run += c;
        }
    }
    __syncthreads();
    if (in) {
        const unsigned pos = offs[dgt] + wcnt[w * kDigits + dgt] + (unsigned)below;
        b.keys[src ^ 1][pos] = key;
        b.ids[src ^ 1][pos] = idv;
    }
}

__global__ void __launch_bounds__(256) rsort_out_kernel(int n, int n_ids, SortBufs b, int *__restrict__ out_ids,
                                                        long long *__restrict__ out_counts) {
    __shared__ unsigned gs[kPasses * kDigits];
    stage_totals<256>(b.gtot, gs);
    const int src = source_buffer(gs, kPasses, n);
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j < n_ids) out_ids[j] = b.ids[src][j];
    if (out_counts != nullptr && j < n) out_counts[j] = (long long)b.keys[src][j];
}

}  // namespace

// sc: counts sorted descending.  out[0] = k, out[1] = mass of the k largest counts, out[2] = total mass.
//   mode 0: smallest k >= 1 with S_k >= ceil(P * total);  mode 1: k = #{c >= f_min}.
// Two launches over the whole device, one workgroup per 1024 counts: the first writes each workgroup's sum
// (and clears `out`), the second lets every workgroup place itself in the running mass.
__global__ void __launch_bounds__(kRankSortThreads) choose_sum_kernel(const long long *__restrict__ sc, int V,
                                                                      long long *__restrict__ bsum,
                                                                      long long *__restrict__ out) {
    __shared__ long long wsum[kSortWaves];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int j = blockIdx.x * kRankSortThreads + tid;
    long long s = j < V ? sc[j] : 0;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) wsum[w] = s;
    __syncthreads();
    if (tid == 0) {
        long long t = 0;
        for (int q = 0; q < kSortWaves; ++q) t += wsum[q];
        bsum[blockIdx.x] = t;
        if (blockIdx.x == 0) {
            out[0] = 0;
            out[1] = 0;
            out[2] = 0;
        }
    }
}

__global__ void __launch_bounds__(kRankSortThreads) choose_k_kernel(const long long *__restrict__ sc, int V, int mode,
                                                                    double P, long long f_min,
                                                                    const long long *__restrict__ bsum,
                                                                    long long *__restrict__ out) {
    __shared__ long long red[2 * kSortWaves];
    __shared__ long long wsum[kSortWaves];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nblk = gridDim.x, blk = blockIdx.x;
    // mass before this workgroup, and in total
    long long before = 0, total = 0;
    for (int x = tid; x < nblk; x += kRankSortThreads) {
        const long long v = bsum[x];
        total += v;
        if (x < blk) before += v;
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        before += __shfl_xor(before, o);
        total += __shfl_xor(total, o);
    }
    if (lane == 0) {
        red[w] = before;
        red[kSortWaves + w] = total;
    }
    __syncthreads();
    before = 0;
    total = 0;
    for (int q = 0; q < kSortWaves; ++q) {
        before += red[q];
        total += red[kSortWaves + q];
    }
    const int j = blk * kRankSortThreads + tid;
    const long long c = j < V ? sc[j] : 0;
    if (blk == 0 && tid == 0) out[2] = total;

    if (mode == 0) {
        // one fp64 product, then its ceiling; never above the total (beyond 2^53 tokens the product of P = 1
        // can round up past it, and no prefix would reach it)
        const long long want = (long long)ceil(P * (double)total);
        const long long target = want > total ? total : want;
        // inclusive prefix of c inside the workgroup: wave scan, then the earlier waves' sums
        long long inc = c;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const long long t = __shfl_up(inc, o);
            if (lane >= o) inc += t;
        }
        if (lane == kWave - 1) wsum[w] = inc;
        __syncthreads();
        long long run = before;
        for (int q = 0; q < w; ++q) run += wsum[q];
        const long long upto = run + inc;          // S_{j+1}
        const long long prev = upto - c;           // S_j
        // exactly one element takes the mass from below the target to at least the target
        // (element 0 also when the target is 0: k >= 1)
        if (j < V && upto >= target && (j == 0 || prev < target)) {
            out[0] = j + 1;
            out[1] = upto;
        }
    } else {
        long long kept = (j < V && c >= f_min) ? 1 : 0, cov = kept ? c : 0;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            kept += __shfl_xor(kept, o);
            cov += __shfl_xor(cov, o);
        }
        if (lane == 0 && kept != 0) {
            atomicAdd(reinterpret_cast<unsigned long long *>(&out[0]), (unsigned long long)kept);
            atomicAdd(reinterpret_cast<unsigned long long *>(&out[1]), (unsigned long long)cov);
        }
    }
}

size_t rank_sort_scratch_bytes(int n) {
    const size_t kb = round256((size_t)n * 8), ib = round256((size_t)n * 4);
    const size_t nblk = ((size_t)n + kRankSortThreads - 1) / kRankSortThreads;
    return 2 * kb + 2 * ib + round256(kPasses * kDigits * 4) + round256(kDigits * nblk * 4);
}

// Sorts all n ids by (count desc, id asc); writes the first n_ids of them and, if asked, all sorted counts.
void launch_rank_sort(const long long *counts, int n, void *scratch, int *out_ids, int n_ids, long long *out_counts,
                      hipStream_t st) {
    char *p = static_cast<char *>(scratch);
    const size_t kb = round256((size_t)n * 8), ib = round256((size_t)n * 4);
    const int nblk = (n + kRankSortThreads - 1) / kRankSortThreads;
    SortBufs b;
    b.keys[0] = reinterpret_cast<unsigned long long *>(p);
    b.keys[1] = reinterpret_cast<unsigned long long *>(p + kb);
    b.ids[0] = reinterpret_cast<int *>(p + 2 * kb);
    b.ids[1] = reinterpret_cast<int *>(p + 2 * kb + ib);
    b.gtot = reinterpret_cast<unsigned *>(p + 2 * kb + 2 * ib);
    b.hist = reinterpret_cast<unsigned *>(p + 2 * kb + 2 * ib + round256(kPasses * kDigits * 4));
    hipLaunchKernelGGL(rsort_zero_kernel, dim3(1), dim3(256), 0, st, b.gtot);
    hipLaunchKernelGGL(rsort_init_kernel, dim3(nblk), dim3(kRankSortThreads), 0, st, counts, n, b);
    for (int pass = 0; pass < kPasses; ++pass) {
        hipLaunchKernelGGL(rsort_hist_kernel, dim3(nblk), dim3(kRankSortThreads), 0, st, n, pass, b);
        hipLaunchKernelGGL(rsort_scatter_kernel, dim3(nblk), dim3(kRankSortThreads), 0, st, n, pass, b);
    }
    hipLaunchKernelGGL(rsort_out_kernel, dim3((n + 255) / 256), dim3(256), 0, st, n, n_ids, b, out_ids, out_counts);
}

size_t choose_k_scratch_bytes(int V) {
    return round256((((size_t)V + kRankSortThreads - 1) / kRankSortThreads) * sizeof(long long));
}

void launch_choose_k(const long long *sorted_counts, int V, int mode, double P, long long f_min, void *scratch,
                     long long *out, hipStream_t st) {
    const int nblk = (V + kRankSortThreads - 1) / kRankSortThreads;
    long long *bsum = static_cast<long long *>(scratch);
    hipLaunchKernelGGL(choose_sum_kernel, dim3(nblk), dim3(kRankSortThreads), 0, st, sorted_counts, V, bsum, out);
    hipLaunchKernelGGL(choose_k_kernel, dim3(nblk), dim3(kRankSortThreads), 0, st, sorted_counts, V, mode, P, f_min,
                       bsum, out);
}

}  // namespace vt
