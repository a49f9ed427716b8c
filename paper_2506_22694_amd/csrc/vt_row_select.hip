// Per-row tail of the draft step for many hidden rows (Algorithm 2's drafting lines after the
// projection): given the raw trimmed logits z[i, 0..k) of a hidden row, its log-sum-exp, its m best
// logits (equal logits -> lower target id) and their target ids.
//
// With tens or hundreds of hidden rows the per-tile candidate lists of the fused path grow to
// megabytes and their selection rounds dominate; it is cheaper to let the matrix-core kernel store
// the logits (n * k * 4 bytes, written once, read back from the L2) and give every hidden row a
// workgroup of its own:
//   pass 1  every thread (1024 per row) folds its share of the row into (max, sum-exp) and keeps its largest logit;
//   T       a threshold that at least m logits reach, from the lanes' maxima (bit-serial selection inside each wave),
//           so the m best logits are all >= T;
//   pass 2  logits >= T become candidate keys in LDS (typically a few dozen), ranked by counting;
//   if more than 1024 logits reach T (massive ties, e.g. h = 0) the m best are extracted one by one.
#include "vt_device.h"
#include "vt_step.h"

namespace vt {

namespace {

constexpr int kRowThreads = 1024;
constexpr int kRowWaves = kRowThreads / kWave;
constexpr int kRowMaxCand = 1024;

__device__ __forceinline__ float block_sum_f32(float v, float *red, int lane, int w) {
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) red[w] = v;
    __syncthreads();
    float r = 0.f;
#pragma unroll
    for (int q = 0; q < kRowWaves; ++q) r += red[q];     // fixed order: reproducible
    return r;
}
__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long *red, int lane,
                                                            int w) {
    v = wave_max_u64(v);
    __syncthreads();
    if (lane == 0) red[w] = v;
    __syncthreads();
    unsigned long long r = red[0];
#pragma unroll
    for (int q = 1; q < kRowWaves; ++q) r = red[q] > r ? red[q] : r;
    return r;
}

}  // namespace

// Values of one thread for one stretch of kRowThreads * kRowVals logits: v[u] = z[base + u * kRowThreads + tid]
// (-inf past the end).  All loads are issued before the first use.
constexpr int kRowVals = 32;
constexpr int kRowSpan = kRowThreads * kRowVals;     // 32768 logits per stretch

// VEC: four consecutive logits per load (k a multiple of 4, row 16-byte aligned): thread t's value u is logit
// base + 4 * ((u / 4) * kRowThreads + t) + u % 4; otherwise logit base + u * kRowThreads + t.
template <bool VEC>
__device__ __forceinline__ int stretch_index(int base, int u, int tid) {
    return VEC ? base + 4 * ((u >> 2) * kRowThreads + tid) + (u & 3) : base + u * kRowThreads + tid;
}
template <bool VEC>
__device__ __forceinline__ void load_stretch(const float *__restrict__ zr, int base, int k, int tid,
                                             float (&v)[kRowVals]) {
    if constexpr (VEC) {
#pragma unroll
        for (int q = 0; q < kRowVals / 4; ++q) {
            const int j = base + 4 * (q * kRowThreads + tid);
            float4 t = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (j < k) t = *reinterpret_cast<const float4 *>(zr + j);
            v[4 * q] = t.x;
            v[4 * q + 1] = t.y;
            v[4 * q + 2] = t.z;
            v[4 * q + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int u = 0; u < kRowVals; ++u) {
            const int j = base + u * kRowThreads + tid;
            v[u] = j < k ? zr[j] : -INFINITY;
        }
    }
}

// KEEP: the row fits one stretch (k <= 32768), so its logits stay in registers for the second pass.
template <bool KEEP, bool VEC>
__global__ void __launch_bounds__(kRowThreads) row_select_kernel(const float *__restrict__ z, const int *__restrict__ map,
                                                                 int k, int m, int *__restrict__ out_ids,
                                                                 float *__restrict__ out_logp,
                                                                 float *__restrict__ out_lse,
                                                                 float *__restrict__ lse_buf) {
    __shared__ float redf[kRowWaves];
    __shared__ unsigned long long red64[kRowWaves];
    __shared__ unsigned tmax[2 * kRowWaves];
    __shared__ unsigned long long cand[kRowMaxCand];
    __shared__ int candj[kRowMaxCand];
    __shared__ unsigned s_ncand;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int i = blockIdx.x;
    const float *zr = z + (size_t)i * k;
    float v[kRowVals];

    // ---- pass 1: (max, sum-exp) and the thread's largest logit
    float lm = -INFINITY, ls = 0.f;
    for (int base = 0; base < k; base += kRowSpan) {
        load_stretch<VEC>(zr, base, k, tid, v);
        float cm = v[0];
#pragma unroll
        for (int u = 1; u < kRowVals; ++u) cm = fmaxf(cm, v[u]);
        const float mn = fmaxf(lm, cm);
        if (mn != -INFINITY) {
            float cs = 0.f;
#pragma unroll
            for (int u = 0; u < kRowVals; ++u) cs += __expf(v[u] - mn);     // exp(-inf) = 0 past the end
            ls = ls * __expf(lm - mn) + cs;
            lm = mn;
        }
    }
    // ---- one exchange through LDS gives the row maximum M and the threshold T, a value that at least m logits
    // reach: every wave finds the ceil(m / 16)-th largest of its lanes' maxima (the wave maximum itself for
    // m <= 16, otherwise bit by bit with ballots); each wave's share then holds that many logits >= its value,
    // so the smallest of the sixteen values is reached by at least 16 * ceil(m / 16) >= m logits.  (Lanes
    // without an element hold the lowest code.)
    const unsigned mine = lm == -INFINITY ? 0u : orderable_f32(lm);
    const unsigned wtop = wave_max_u32(mine);
    unsigned Tw = wtop;
    int need = (m + kRowWaves - 1) / kRowWaves;
    if (need > 1) {
        Tw = 0u;
        unsigned long long alive = ~0ull;
        for (int b = 31; b >= 0; --b) {
            const unsigned long long ones = __ballot((mine >> b) & 1u) & alive;
            const int c = __popcll(ones);
            if (c >= need) {
                alive = ones;
                Tw |= 1u << b;
            } else {
                need -= c;
                alive &= ~ones;
            }
        }
    }
    if (tid == 0) s_ncand = 0u;
    if (lane == 0) {
        tmax[w] = Tw;
        tmax[kRowWaves + w] = wtop;
    }
    __syncthreads();
    unsigned T = tmax[0], Mo = tmax[kRowWaves];
#pragma unroll
    for (int q = 1; q < kRowWaves; ++q) {
        T = tmax[q] < T ? tmax[q] : T;
        Mo = tmax[kRowWaves + q] > Mo ? tmax[kRowWaves + q] : Mo;
    }
    const float M = from_orderable_f32(Mo);      // k >= 1: some lane holds an element
    const float S = block_sum_f32(lm == -INFINITY ? 0.f : ls * __expf(lm - M), redf, lane, w);
    const float lse = M + __logf(S);
    // compared as a float below (the order code is monotone; code 0 = no element maps to "everything passes")
    const float Tf = T == 0u ? -INFINITY : from_orderable_f32(T);

    // ---- pass 2: every logit >= T is a candidate
    for (int base = 0; base < k; base += kRowSpan) {
        if (!KEEP) load_stretch<VEC>(zr, base, k, tid, v);
#pragma unroll
        for (int u = 0; u < kRowVals; ++u) {
            const int j = stretch_index<VEC>(base, u, tid);
            if (j < k && v[u] >= Tf) {
                // logit and position now, the target id later: a load from the map here would put a trip to
                // memory behind every candidate a wave finds, one after the other
                const unsigned slot = atomicAdd(&s_ncand, 1u);
                if (slot < (unsigned)kRowMaxCand) {
                    cand[slot] = (unsigned long long)__float_as_uint(v[u]);
                    candj[slot] = j;
                }
            }
        }
    }
    __syncthreads();
    const int ncand = (int)s_ncand;
    if (ncand <= kRowMaxCand) {
        // the candidates' target ids, all requested at once
        for (int c = tid; c < ncand; c += kRowThreads)
            cand[c] = make_key(__uint_as_float((unsigned)cand[c]), map[candj[c]]);
        __syncthreads();
        // rank by counting: keys are distinct (distinct target ids)
        for (int c = tid; c < ncand; c += kRowThreads) {
            const unsigned long long key = cand[c];
            unsigned above = 0;
            int x = 0;
            for (; x + 8 <= ncand; x += 8) {
                unsigned long long t[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) t[u] = cand[x + u];
#pragma unroll
                for (int u = 0; u < 8; ++u) above += t[u] > key ? 1u : 0u;
            }
            for (; x < ncand; ++x) above += cand[x] > key ? 1u : 0u;
            if ((int)above < m) {
                out_ids[(size_t)i * m + above] = key_id(key);
                out_logp[(size_t)i * m + above] = key_logit(key) - lse;
            }
        }
    } else {
        // massive ties: take the best remaining key, m times (each round re-reads the row from the L2)
        unsigned long long prev = ~0ull;
        for (int r = 0; r < m; ++r) {
            unsigned long long best = kNoKey;
            for (int base = 0; base < k; base += kRowSpan) {
                if (!KEEP) load_stretch<VEC>(zr, base, k, tid, v);
#pragma unroll
                for (int u = 0; u < kRowVals; ++u) {
                    const int j = stretch_index<VEC>(base, u, tid);
                    if (j < k && v[u] >= Tf) {
                        const unsigned long long key = make_key(v[u], map[j]);
                        if (key < prev && key > best) best = key;
                    }
                }
            }
            best = block_max_u64(best, red64, lane, w);
            if (tid == 0) {
                out_ids[(size_t)i * m + r] = key_id(best);
                out_logp[(size_t)i * m + r] = key_logit(best) - lse;
            }
            prev = best;
        }
    }
    if (tid == 0) {
        lse_buf[i] = lse;
        if (out_lse != nullptr) out_lse[i] = lse;
    }
}

void launch_row_select(const float *z, const int *map, int n, int k, int m, int *out_ids, float *out_logp,
                       float *out_lse, float *lse_buf, hipStream_t st) {
    const bool vec = (k & 3) == 0 && (reinterpret_cast<uintptr_t>(z) & 15) == 0;
    const bool keep = k <= kRowSpan;
    auto kern = keep ? (vec ? row_select_kernel<true, true> : row_select_kernel<true, false>)
                     : (vec ? row_select_kernel<false, true> : row_select_kernel<false, false>);
    hipLaunchKernelGGL(kern, dim3(n), dim3(kRowThreads), 0, st, z, map, k, m, out_ids, out_logp, out_lse, lse_buf);
}

}  // namespace vt
