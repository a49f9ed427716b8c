// Frequency-rank order and the alternative choices of k (Sec. 3.2: besides a fixed k, Top-P over
// the counts or a minimum-frequency threshold select the trimmed vocabulary).
//
// rank_sort_kernel: stable LSD radix sort of (count, id) pairs by count, descending, 4 bits per
//   pass; the ids arrive ascending, so equal counts stay in ascending-id order -- the order in
//   which Top-K(c, k) takes ids, every prefix being the selection for a smaller k.  Only as many
//   passes as the largest count has hex digits (6 for 10^7 calibration tokens).  One workgroup;
//   a wave owns a contiguous segment and walks it 64 elements at a time, so loads are coalesced
//   and "earlier in the input" is (iteration, lane) order: lanes with equal digits find each other
//   with five ballots and rank themselves with a population count.
// choose_k_kernel: prefix sums over the sorted counts; the smallest prefix whose mass reaches
//   ceil(P * total), or the number of counts >= f_min.
#include "vt_build.h"
#include "vt_device.h"

namespace vt {

namespace {

constexpr int kSortWaves = kRankSortThreads / kWave;   // 16
constexpr int kRankUnroll = 8;                         // segment iterations whose loads are in flight together

// lanes of the wave whose `dgt` (0..16) equals this lane's
__device__ __forceinline__ unsigned long long match_digit(int dgt) {
    unsigned long long m = ~0ull;
#pragma unroll
    for (int b = 0; b < 5; ++b) {
        const bool bit = (dgt >> b) & 1;
        const unsigned long long B = __ballot(bit);
        m &= bit ? B : ~B;
    }
    return m;
}
__device__ __forceinline__ int lanes_below(unsigned long long m) {
    return (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
}

// The ping-pong buffers are written by one wave and read by another in the next pass: device-scope
// relaxed atomics go to the L2 both ways, so no stale line of this CU's vector cache is ever read.
__device__ __forceinline__ unsigned long long ld64(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld32(const int *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st64(unsigned long long *p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st32(int *p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

}  // namespace

__global__ void __launch_bounds__(kRankSortThreads) rank_sort_kernel(const long long *__restrict__ counts,
                                                                     const int *__restrict__ ids_in, int n,
                                                                     unsigned long long *kA, unsigned long long *kB,
                                                                     int *iA, int *iB, int *__restrict__ out_ids,
                                                                     long long *__restrict__ out_counts) {
    __shared__ unsigned cnt_s[kSortWaves * 16];
    __shared__ unsigned long long s_max[kSortWaves];
    volatile unsigned *cnt = cnt_s;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int seg = ((n + kSortWaves - 1) / kSortWaves + kWave - 1) / kWave * kWave;
    const int s0 = w * seg, s1 = min(n, s0 + seg);

    unsigned long long mx = 0;
    for (int j = s0 + lane; j < s1; j += kWave) {
        const int id = ids_in != nullptr ? ids_in[j] : j;
        const unsigned long long c = (unsigned long long)counts[id];
        st64(kA + j, c);
        st32(iA + j, id);
        mx = c > mx ? c : mx;
    }
    mx = wave_max_u64(mx);
    if (lane == 0) s_max[w] = mx;
    __syncthreads();
    mx = 0;
    for (int q = 0; q < kSortWaves; ++q) mx = s_max[q] > mx ? s_max[q] : mx;
    const int nbits = mx == 0 ? 0 : 64 - __clzll((long long)mx);
    const int npass = (nbits + 3) / 4;

    unsigned long long *ks = kA, *kd = kB;
    int *is = iA, *id_ = iB;
    for (int p = 0; p < npass; ++p) {
        const int sh = 4 * p;
        if (lane < 16) cnt[w * 16 + lane] = 0u;
        __builtin_amdgcn_wave_barrier();
        // ---- how many elements of each digit this wave holds (digit 0 = largest hex digit: descending order)
        // kRankUnroll iterations' keys are requested together: the device-scope loads take about a
        // microsecond each and nothing else hides them
        for (int j0 = s0; j0 < s1; j0 += kRankUnroll * kWave) {
            unsigned long long keyu[kRankUnroll];
#pragma unroll
            for (int u = 0; u < kRankUnroll; ++u) {
                const int j = j0 + u * kWave + lane;
                keyu[u] = j < s1 ? ld64(ks + j) : 0ull;
            }
#pragma unroll
            for (int u = 0; u < kRankUnroll; ++u) {
                const int j = j0 + u * kWave + lane;
                if (j0 + u * kWave < s1) {                      // wave-uniform
                    const bool in = j < s1;
                    const int dgt = in ? 15 - (int)((keyu[u] >> sh) & 15ull) : 16;
                    const unsigned long long m = match_digit(dgt);
                    if (in && lanes_below(m) == 0) cnt[w * 16 + dgt] = cnt[w * 16 + dgt] + (unsigned)__popcll(m);
                }
            }
        }
        __syncthreads();
        // ---- exclusive prefix over (digit, wave): the first output slot of every (wave, digit) run
        if (w == 0) {
            const int dgt = lane >> 2, wv0 = (lane & 3) * 4;
            unsigned v[4], s = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                v[q] = cnt[(wv0 + q) * 16 + dgt];
                s += v[q];
            }
            unsigned inc = s;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const unsigned t = __shfl_up(inc, o);
                if (lane >= o) inc += t;
            }
            unsigned run = inc - s;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                cnt[(wv0 + q) * 16 + dgt] = run;
                run += v[q];
            }
        }
        __syncthreads();
        // ---- stable scatter
        for (int j0 = s0; j0 < s1; j0 += kRankUnroll * kWave) {
            unsigned long long keyu[kRankUnroll];
            int idu[kRankUnroll];
#pragma unroll
            for (int u = 0; u < kRankUnroll; ++u) {
                const int j = j0 + u * kWave + lane;
                keyu[u] = j < s1 ? ld64(ks + j) : 0ull;
                idu[u] = j < s1 ? ld32(is + j) : 0;
            }
#pragma unroll
            for (int u = 0; u < kRankUnroll; ++u) {
                const int j = j0 + u * kWave + lane;
                if (j0 + u * kWave < s1) {                      // wave-uniform
                    const bool in = j < s1;
                    const int dgt = in ? 15 - (int)((keyu[u] >> sh) & 15ull) : 16;
                    const unsigned long long m = match_digit(dgt);
                    const int below = lanes_below(m);
                    const unsigned base = in ? cnt[w * 16 + dgt] : 0u;
                    __builtin_amdgcn_wave_barrier();       // every lane has read its base before a leader moves it
                    if (in) {
                        st64(kd + base + below, keyu[u]);
                        st32(id_ + base + below, idu[u]);
                        if (below == 0) cnt[w * 16 + dgt] = base + (unsigned)__popcll(m);
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            }
        }
        __syncthreads();   // the pass is complete (and visible to the whole workgroup) before the next reads it
        unsigned long long *tk = ks;
        ks = kd;
        kd = tk;
        int *ti = is;
        is = id_;
        id_ = ti;
    }
    for (int j = tid; j < n; j += kRankSortThreads) {
        out_ids[j] = ld32(is + j);
        if (out_counts != nullptr) out_counts[j] = (long long)ld64(ks + j);
    }
}

// sc: counts sorted descending.  out[0] = k, out[1] = mass of the k largest counts, out[2] = total mass.
//   mode 0: smallest k >= 1 with S_k >= ceil(P * total);  mode 1: k = #{c >= f_min}.
__global__ void __launch_bounds__(kRankSortThreads) choose_k_kernel(const long long *__restrict__ sc, int V, int mode,
                                                                    double P, long long f_min,
                                                                    long long *__restrict__ out) {
    __shared__ long long wsum[kSortWaves], wkept[kSortWaves];
    __shared__ long long s_k, s_cov;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int seg = ((V + kSortWaves - 1) / kSortWaves + kWave - 1) / kWave * kWave;
    const int s0 = w * seg, s1 = min(V, s0 + seg);
    long long s = 0;
    for (int j = s0 + lane; j < s1; j += kWave) s += sc[j];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) wsum[w] = s;
    if (tid == 0) {
        s_k = -1;
        s_cov = 0;
    }
    __syncthreads();
    long long total = 0, before = 0;
    for (int q = 0; q < kSortWaves; ++q) {
        if (q < w) before += wsum[q];
        total += wsum[q];
    }
    if (mode == 0) {
        long long target = (long long)ceil(P * (double)total);     // one fp64 product, then its ceiling
        // exactly one wave holds the element that takes the running mass from below the target to at least
        // the target (wave 0 also when the target is 0: k >= 1)
        const bool mine = (w == 0 || before < target) && before + wsum[w] >= target && s1 > s0;
        if (mine) {
            long long run = before;
            for (int j0 = s0; j0 < s1; j0 += kWave) {
                const int j = j0 + lane;
                const long long c = j < s1 ? sc[j] : 0;
                long long inc = c;
#pragma unroll
                for (int o = 1; o < kWave; o <<= 1) {
                    const long long t = __shfl_up(inc, o);
                    if (lane >= o) inc += t;
                }
                const bool hit = j < s1 && run + inc >= target;
                const unsigned long long b = __ballot(hit);
                if (b != 0ull) {
                    const int first = __ffsll((long long)b) - 1;
                    if (lane == first) {
                        s_k = j + 1;
                        s_cov = run + inc;
                    }
                    break;
                }
                run += __shfl(inc, kWave - 1);
            }
        }
    } else {
        // counts are sorted: k = index of the first count below f_min
        long long kept = 0, cov = 0;
        for (int j = s0 + lane; j < s1; j += kWave) {
            const long long c = sc[j];
            if (c >= f_min) {
                kept += 1;
                cov += c;
            }
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            kept += __shfl_xor(kept, o);
            cov += __shfl_xor(cov, o);
        }
        if (lane == 0) {
            atomicAdd(reinterpret_cast<unsigned long long *>(&s_cov), (unsigned long long)cov);
            wkept[w] = kept;
        }
    }
    __syncthreads();
    if (tid == 0) {
        if (mode == 0) {
            out[0] = s_k;
            out[1] = s_cov;
        } else {
            long long k = 0;
            for (int q = 0; q < kSortWaves; ++q) k += wkept[q];
            out[0] = k;
            out[1] = s_cov;
        }
        out[2] = total;
    }
}

void launch_rank_sort(const long long *counts, const int *ids_in, int n, void *scratch, int *out_ids,
                      long long *out_counts, hipStream_t st) {
    char *p = static_cast<char *>(scratch);
    const size_t kb = ((size_t)n * 8 + 255) / 256 * 256, ib = ((size_t)n * 4 + 255) / 256 * 256;
    unsigned long long *kA = reinterpret_cast<unsigned long long *>(p);
    unsigned long long *kB = reinterpret_cast<unsigned long long *>(p + kb);
    int *iA = reinterpret_cast<int *>(p + 2 * kb);
    int *iB = reinterpret_cast<int *>(p + 2 * kb + ib);
    hipLaunchKernelGGL(rank_sort_kernel, dim3(1), dim3(kRankSortThreads), 0, st, counts, ids_in, n, kA, kB, iA, iB,
                       out_ids, out_counts);
}

size_t rank_sort_scratch_bytes(int n) {
    const size_t kb = ((size_t)n * 8 + 255) / 256 * 256, ib = ((size_t)n * 4 + 255) / 256 * 256;
    return 2 * kb + 2 * ib;
}

void launch_choose_k(const long long *sorted_counts, int V, int mode, double P, long long f_min, long long *out,
                     hipStream_t st) {
    hipLaunchKernelGGL(choose_k_kernel, dim3(1), dim3(kRankSortThreads), 0, st, sorted_counts, V, mode, P, f_min, out);
}

}  // namespace vt
