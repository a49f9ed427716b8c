// Algorithm 1 (Count Token Frequencies): c[t] += 1 for every token id of the stream.
//
// The V counters do not fit one CU's LDS as 32-bit words (V = 128256 -> 513 KB), so the bins
// are 16 bits wide, two per LDS word, the vocabulary is cut into ranges of 65536 bins (128 KiB of
// LDS; two ranges for V = 128256) and the id stream into chunks.  Workgroup (chunk, range) reads
// its chunk with 16-byte loads, counts the ids that fall into its range with LDS atomics (no
// global atomic sees the Zipf-hot ids more than once per 32768 occurrences), and writes its
// private histogram to scratch.  A second kernel sums the chunk histograms into the caller's
// int64 counters.  Ids outside [0, V) are skipped and tallied.
//
// A 16-bit bin never holds more than 15 bits for long: the increment that sets bit 15 (it sees the
// old value 0x7FFF) takes 32768 back out of the bin and adds them to the result counter directly.
// Between that increment and its subtraction the bin can only grow by the increments in flight in
// the workgroup (a few thousand at most), far from 65536, so a bin never carries into its
// neighbour in the same word, whatever the id distribution.
#include "vt_build.h"
#include "vt_device.h"
#include "vt_launch.h"
#include <type_traits>

namespace vt {

int hist_num_ranges(int V) { return (V + kHistBinsPerBlock - 1) / kHistBinsPerBlock; }

int hist_num_chunks(int64_t n_ids, int V) {
    // at least 64K ids per chunk so that zeroing and flushing 128 KiB of LDS pays off; chunks x ranges = one
    // round of workgroups over the 256 CUs
    int cap = kHistBlocks / hist_num_ranges(V);
    if (cap < 1) cap = 1;
    int64_t c = (n_ids + (1 << 16) - 1) >> 16;
    if (c < 1) c = 1;
    if (c > cap) c = cap;
    return (int)c;
}

// `head` ids (fewer than one 16-byte vector) precede the first 16-byte aligned id.
template <bool IDS64>
__global__ void __launch_bounds__(kHistThreads) hist_partial_kernel(const void *__restrict__ ids_v, long long n_ids,
                                                                    int head, int V, int nchunks,
                                                                    unsigned *__restrict__ partial,
                                                                    unsigned long long *__restrict__ counts,
                                                                    unsigned long long *__restrict__ n_invalid) {
    extern __shared__ __align__(16) unsigned words[];     // two 16-bit bins per word
    const int chunk = blockIdx.x, range = blockIdx.y;
    const int lo = range * kHistBinsPerBlock;
    const int nb = min(kHistBinsPerBlock, V - lo);
    const int nw = (nb + 1) >> 1;
    for (int b = threadIdx.x; b < nw; b += kHistThreads) words[b] = 0u;
    __syncthreads();

    // chunk boundaries in units of 16-byte vectors (4 int32 or 2 int64), tail handled by the last chunk
    constexpr int IPV = IDS64 ? 2 : 4;
    constexpr int IDB = IDS64 ? 8 : 4;
    const long long nvec = (n_ids - head) / IPV;
    const long long v0 = nvec * chunk / nchunks, v1 = nvec * (chunk + 1) / nchunks;
    unsigned invalid = 0;
    // One id.  (The scalar head and tail of the stream.)
    auto tally = [&](long long t) {
        if ((unsigned long long)t >= (unsigned long long)V) {
            invalid += 1u;
        } else {
            const unsigned b = (unsigned)((int)t - lo);
            if (b < (unsigned)nb) {
                const unsigned sh = (b & 1u) << 4;
                const unsigned old = atomicAdd(&words[b >> 1], 1u << sh);
                if (((old >> sh) & 0xFFFFu) == 0x7FFFu) {
                    // this increment set bit 15: 32768 occurrences move from the bin to the result counter
                    atomicSub(&words[b >> 1], 0x8000u << sh);
                    atomicAdd(&counts[t], 32768ull);
                }
            }
        }
    };
    // The ids of NV 16-byte vectors: all their LDS atomics are issued before the first result is looked at -- a
    // wave that waited for every atomic's return before the next id spent most of its time in that wait -- and the
    // rare increment that sets bit 15 is handled behind one test for the whole batch.
    constexpr int IPV0 = IDS64 ? 2 : 4;
    auto tally_ids = [&](auto ncount, const long long *t) {
        constexpr int N = decltype(ncount)::value;
        // ids outside [0, V): rare, so one test for the batch (the largest id as an unsigned number) and the count
        // behind it; only the workgroups of range 0 report them
        if (range == 0) {
            bool some;
            if constexpr (IDS64) {
                unsigned long long mx = (unsigned long long)t[0];
#pragma unroll
                for (int q = 1; q < N; ++q) mx = (unsigned long long)t[q] > mx ? (unsigned long long)t[q] : mx;
                some = mx >= (unsigned long long)V;
            } else {
                unsigned mx = (unsigned)(int)t[0];       // a negative id is a large unsigned number
#pragma unroll
                for (int q = 1; q < N; ++q) mx = (unsigned)(int)t[q] > mx ? (unsigned)(int)t[q] : mx;
                some = mx >= (unsigned)V;
            }
            if (some) {
#pragma unroll
                for (int q = 0; q < N; ++q) invalid += (unsigned long long)t[q] >= (unsigned long long)V ? 1u : 0u;
            }
        }
        unsigned b[N], inc[N], old[N];
        bool in[N];
#pragma unroll
        for (int q = 0; q < N; ++q) {
            // bin inside this range; an id outside [lo, lo + nb) -- a negative one too, V < 2^31 -- wraps far past nb
            // (a 64-bit id is first checked as a whole: its low half alone could land anywhere)
            b[q] = (unsigned)((int)t[q] - lo);
            in[q] = b[q] < (unsigned)nb && (!IDS64 || (unsigned long long)t[q] < (unsigned long long)V);
            inc[q] = 1u + (b[q] & 1u) * 0xFFFFu;        // 1 for the low half of the word, 0x10000 for the high one
            old[q] = 0u;
        }
#pragma unroll
        for (int q = 0; q < N; ++q) {
            if (in[q]) old[q] = atomicAdd(&words[b[q] >> 1], inc[q]);
        }
        // the increment that found 0x7FFF in its bin set bit 15
        bool spill = false;
#pragma unroll
        for (int q = 0; q < N; ++q) spill |= in[q] && (old[q] & (inc[q] * 0x7FFFu)) == inc[q] * 0x7FFFu;
        if (spill) {
#pragma unroll
            for (int q = 0; q < N; ++q) {
                if (in[q] && (old[q] & (inc[q] * 0x7FFFu)) == inc[q] * 0x7FFFu) {
                    // 32768 occurrences move from the bin to the result counter
                    atomicSub(&words[b[q] >> 1], inc[q] * 0x8000u);
                    atomicAdd(&counts[t[q]], 32768ull);
                }
            }
        }
    };
    const u32x4 *vp = reinterpret_cast<const u32x4 *>(static_cast<const char *>(ids_v) + (size_t)head * IDB);
    auto unpack = [&](const u32x4 q, long long *t) {
        if constexpr (IDS64) {
            t[0] = (long long)(((unsigned long long)q.y << 32) | q.x);
            t[1] = (long long)(((unsigned long long)q.w << 32) | q.z);
        } else {
            t[0] = (long long)(int)q.x;
            t[1] = (long long)(int)q.y;
            t[2] = (long long)(int)q.z;
            t[3] = (long long)(int)q.w;
        }
    };
    auto tally_vec = [&](const u32x4 q) {
        long long t[IPV0];
        unpack(q, t);
        tally_ids(std::integral_constant<int, IPV0>{}, t);
    };
    auto tally_vec2 = [&](const u32x4 q0, const u32x4 q1) {
        long long t[2 * IPV0];
        unpack(q0, t);
        unpack(q1, t + IPV0);
        tally_ids(std::integral_constant<int, 2 * IPV0>{}, t);
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
        static_assert(kHistUnroll % 2 == 0, "vectors are counted in pairs");
#pragma unroll
        for (int u = 0; u < kHistUnroll; u += 2) tally_vec2(q[u], q[u + 1]);
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
    // rows of the scratch are (V rounded up to even) 16-bit bins long: every range starts on a word
    unsigned *dst = partial + (((size_t)chunk * (size_t)((V + 1) & ~1) + lo) >> 1);
    for (int b = threadIdx.x; b < nw; b += kHistThreads) dst[b] = words[b];
    // every range-workgroup of a chunk sees the same invalid ids: only range 0 reports them
    if (n_invalid != nullptr && range == 0) {
        const int tot = wave_sum_i32((int)invalid);
        if (lane_id() == 0 && tot != 0) atomicAdd(n_invalid, (unsigned long long)tot);
    }
}

// A workgroup sums 64 words (128 neighbouring bins) over the chunks: wave g takes the chunks g, g + 4, ..
// (a load instruction reads 256 consecutive bytes of one chunk's row), the four partial sums meet in LDS.
__global__ void __launch_bounds__(256) hist_reduce_kernel(const unsigned *__restrict__ partial, int nchunks, int V,
                                                          long long *__restrict__ counts) {
    __shared__ long long part[3][2][kWave];
    const int lane = (int)threadIdx.x & 63, g = (int)threadIdx.x >> 6;
    const int wi = blockIdx.x * kWave + lane;
    const int Vw = (V + 1) >> 1;                   // words per scratch row
    long long s0 = 0, s1 = 0;
    if (wi < Vw) {
        int c = g;
        for (; c + 12 < nchunks; c += 16) {
            unsigned t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u] = partial[(size_t)(c + 4 * u) * Vw + wi];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                s0 += (long long)(t[u] & 0xFFFFu);
                s1 += (long long)(t[u] >> 16);
            }
        }
        for (; c < nchunks; c += 4) {
            const unsigned t = partial[(size_t)c * Vw + wi];
            s0 += (long long)(t & 0xFFFFu);
            s1 += (long long)(t >> 16);
        }
    }
    if (g > 0) {
        part[g - 1][0][lane] = s0;
        part[g - 1][1][lane] = s1;
    }
    __syncthreads();
    if (g == 0 && wi < Vw) {
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            s0 += part[q][0][lane];
            s1 += part[q][1][lane];
        }
        counts[2 * wi] += s0;
        if (2 * wi + 1 < V) counts[2 * wi + 1] += s1;
    }
}

hipError_t launch_count_tokens(const void *ids, bool ids64, int64_t n_ids, int V, long long *counts,
                         unsigned long long *n_invalid, unsigned *partial, hipStream_t st) {
    const int nchunks = hist_num_chunks(n_ids, V);
    const int nranges = hist_num_ranges(V);
    const size_t lds = (size_t)kHistBinsPerBlock * sizeof(unsigned short);
    static LdsLimitOnce lds_limit;
    hipError_t e = allow_dynamic_lds(lds_limit, {reinterpret_cast<const void *>(hist_partial_kernel<false>),
                                                 reinterpret_cast<const void *>(hist_partial_kernel<true>)}, (int)lds);
    if (e != hipSuccess) return e;
    dim3 grid(nchunks, nranges);
    // ids before the first 16-byte boundary are counted one by one
    const int idb = ids64 ? 8 : 4;
    const uintptr_t mis = reinterpret_cast<uintptr_t>(ids) & 15u;
    long long head = mis ? (long long)((16 - mis) / idb) : 0;
    if (head > n_ids) head = n_ids;
    if (ids64)
        hipLaunchKernelGGL(hist_partial_kernel<true>, grid, dim3(kHistThreads), lds, st, ids, (long long)n_ids,
                           (int)head, V, nchunks, partial, reinterpret_cast<unsigned long long *>(counts), n_invalid);
    else
        hipLaunchKernelGGL(hist_partial_kernel<false>, grid, dim3(kHistThreads), lds, st, ids, (long long)n_ids,
                           (int)head, V, nchunks, partial, reinterpret_cast<unsigned long long *>(counts), n_invalid);
    hipLaunchKernelGGL(hist_reduce_kernel, dim3(((V + 1) / 2 + kWave - 1) / kWave), dim3(256), 0, st, partial, nchunks, V,
                       counts);
    return hipGetLastError();
}

}  // namespace vt
