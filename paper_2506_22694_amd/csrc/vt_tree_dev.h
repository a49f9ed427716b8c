// "The K largest of N keys" for a workgroup of T threads and N <= T candidates, by counting: every
// candidate finds its rank as the number of keys above its own.  The keys sit in LDS and every lane
// of a wave reads the same one (a broadcast, no bank conflicts); T / N2 threads share one
// candidate's scan.  Shared by the stand-alone tree kernels and by the draft step's fused tree level.
#pragma once
#include "vt_device.h"
#include "vt_tree.h"

namespace vt {

// COHERENT: the inputs were written earlier in this same kernel by other waves of this workgroup
// (fused tree level), so they are read with device-scope loads that do not trust this CU's vector cache.
template <bool COHERENT>
__device__ __forceinline__ unsigned long long tree_key(const TreeArgs &a, int c) {
    if (c >= a.N) return kNoKey;
    float s;
    if constexpr (COHERENT) {
        s = __uint_as_float(__hip_atomic_load(reinterpret_cast<const unsigned *>(a.vals) + c, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT));
    } else {
        s = a.vals[c];
    }
    if (a.parent_cum != nullptr) s = __fadd_rn(a.parent_cum[c / a.m], s);   // one fp32 addition
    return make_key(s, c);
}

// The token of candidate c (c itself without an id table); requested together with the candidate's score so
// that the two round trips overlap.
template <bool COHERENT>
__device__ __forceinline__ int tree_token(const TreeArgs &a, int c) {
    if (c >= a.N || a.ids == nullptr || a.out_token == nullptr) return c;
    if constexpr (COHERENT)
        return __hip_atomic_load(a.ids + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
        return a.ids[c];
}

__device__ __forceinline__ void tree_emit(const TreeArgs &a, int slot, unsigned long long key, int tok) {
    const int c = key_id(key);
    a.out_a[slot] = a.parent_cum != nullptr ? c / a.m : c;
    if (a.out_token != nullptr) a.out_token[slot] = tok;
    if (a.out_score != nullptr) a.out_score[slot] = key_logit(key);
}

// keys: N2 u64, cnt: N2 u32, wave_tot: T / 64 ints, all in LDS and free for use.  N2 = power of two with
// 64 <= N2 <= T and a.N <= N2.  Every thread of the workgroup must call; contains barriers.
template <int T, bool COHERENT>
__device__ __forceinline__ void tree_select_by_count(const TreeArgs &a, int N2, unsigned long long *keys,
                                                     unsigned *cnt, int *wave_tot) {
    const int tid = threadIdx.x;
    int tok = 0;           // threads 0 .. N2-1 own candidate tid
    if (tid < N2) {
        tok = tree_token<COHERENT>(a, tid);
        keys[tid] = tree_key<COHERENT>(a, tid);
        cnt[tid] = 0u;
    }
    __syncthreads();
    const int c = tid & (N2 - 1), part = tid / N2, parts = T / N2;
    const int j0 = (int)((long long)a.N * part / parts), j1 = (int)((long long)a.N * (part + 1) / parts);
    const unsigned long long mine = keys[c];
    unsigned above = 0;
    int j = j0;
    for (; j + 8 <= j1; j += 8) {      // eight LDS reads in flight: the loop is latency-bound otherwise
        unsigned long long t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = keys[j + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) above += t[u] > mine ? 1u : 0u;
    }
    for (; j < j1; ++j) above += keys[j] > mine ? 1u : 0u;
    if (parts > 1) {
        if (above != 0u) atomicAdd(&cnt[c], above);
        __syncthreads();
        above = cnt[c];
    }
    // threads 0 .. N2-1 (whole waves) own one candidate each
    const bool keep = tid < a.N && (int)above < a.K;
    if (!a.index_order) {
        if (keep) tree_emit(a, (int)above, mine, tok);
        return;
    }
    const unsigned long long bal = __ballot(keep);
    const int lane = tid & 63, w = tid >> 6;
    if (lane == 0) wave_tot[w] = __popcll(bal);
    __syncthreads();
    if (!keep) return;
    int base = 0;
    for (int q = 0; q < w; ++q) base += wave_tot[q];
    const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    tree_emit(a, base + __popcll(bal & below), mine, tok);
}

}  // namespace vt
