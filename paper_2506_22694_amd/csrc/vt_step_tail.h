// Tail of the draft step, shared by its kernels: per-workgroup epilogue
// (log-sum-exp partial + best candidates of a tile of logits), publication,
// election of the last workgroup, and the final cross-workgroup merge
// (lse, top-m, remap to target ids).
#pragma once
#include "vt_device.h"
#include "vt_step.h"

namespace vt {

// ------------------------------------------------------------------ top-L of a wave's candidates
// Every lane holds Q candidates: ord[q] = orderable logit (0 = none), id[q] =
// target id.  L rounds; round r finds the best remaining candidate of the whole
// wave under (logit desc, id asc) and parks it in lane r.  Returns lane r's key.
template <int Q>
__device__ __forceinline__ unsigned long long wave_select_top(unsigned (&ord)[Q], int (&id)[Q], int L, int lane) {
    unsigned res_ord = 0u;
    unsigned res_id = 0u;
    for (int r = 0; r < L; ++r) {
        unsigned bo = ord[0];
#pragma unroll
        for (int q = 1; q < Q; ++q) bo = ord[q] > bo ? ord[q] : bo;
        const unsigned wmax = wave_max_u32(bo);
        unsigned myid = 0xFFFFFFFFu;
        int cnt = 0;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (ord[q] == wmax) {
                myid = (unsigned)id[q] < myid ? (unsigned)id[q] : myid;
                ++cnt;
            }
        }
        // exact ties are rare: one holder -> read its id; otherwise reduce for the lowest id
        const unsigned long long holders = __ballot(cnt > 0);
        const unsigned long long multi = __ballot(cnt > 1);
        unsigned wid;
        if (__popcll(holders) == 1 && multi == 0ull) {
            wid = __builtin_amdgcn_readlane(myid, __ffsll((long long)holders) - 1);
        } else {
            wid = wave_min_u32(myid);
        }
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (ord[q] == wmax && (unsigned)id[q] == wid) ord[q] = 0u;
        }
        if (lane == r) {
            res_ord = wmax;
            res_id = wid;
        }
    }
    return res_ord == 0u ? kNoKey : (((unsigned long long)res_ord << 32) | (unsigned)(~res_id));
}

__device__ __forceinline__ unsigned wave_min_of_group_max_u32(unsigned v, int gsteps);

// The largest value P << 16 such that at least `kth` lanes hold v >= P << 16 (0 if fewer than kth lanes hold anything
// but 0): the upper half of the kth largest v, selected one bit at a time.  All 64 lanes take part.
__device__ __forceinline__ unsigned wave_kth_largest_prefix16(unsigned v, int kth) {
    unsigned T = 0u;
    unsigned long long alive = ~0ull;
    int need = kth;
#pragma unroll
    for (int b = 31; b >= 16; --b) {
        const unsigned long long ones = __ballot((v >> b) & 1u) & alive;
        const int c = __popcll(ones);
        if (c >= need) {
            alive = ones;
            T |= 1u << b;
        } else {
            need -= c;
            alive &= ~ones;
        }
    }
    return T;
}

// ------------------------------------------------------------------ top-L of a wave's candidates, by threshold
// Two candidates per lane (ord = 0: none).  With G = the power of two >= L the lanes form G groups; every
// group's best logit is a different candidate, so at least L candidates reach T = the smallest group maximum
// and the L best are among those that do (about 2 L of 128).  They are compacted into `cand` (wave-private
// LDS, 128 keys) and each finds its rank by counting: no L dependent selection rounds.  Rank r < L is
// published at slot r; slots past the number of candidates get the "no key" value.
__device__ __forceinline__ void wave_publish_top_by_threshold(const unsigned (&ord)[2], const int (&id)[2], int L,
                                                              unsigned long long *cand,
                                                              unsigned long long *__restrict__ pkeys_slot, int lane) {
    const unsigned top = ord[0] > ord[1] ? ord[0] : ord[1];
    unsigned T;
    if (L <= 8) {
        int gsteps = 6;
        while ((kWave >> gsteps) < L) --gsteps;
        T = wave_min_of_group_max_u32(top, gsteps);
    } else {
        T = wave_kth_largest_prefix16(top, L);      // (16 or more groups would pass several times L candidates)
    }
    T = T == 0u ? 1u : T;               // a group without candidates: every real candidate passes
    const bool c0 = ord[0] >= T, c1 = ord[1] >= T;
    const unsigned long long m0 = __ballot(c0), m1 = __ballot(c1);
    const int n0 = __popcll(m0);
    const int ncand = n0 + __popcll(m1);
    const unsigned long long k0 = ((unsigned long long)ord[0] << 32) | (unsigned)(~(unsigned)id[0]);
    const unsigned long long k1 = ((unsigned long long)ord[1] << 32) | (unsigned)(~(unsigned)id[1]);
    if (c0) cand[__builtin_amdgcn_mbcnt_hi((unsigned)(m0 >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m0, 0u))] = k0;
    if (c1)
        cand[n0 + __builtin_amdgcn_mbcnt_hi((unsigned)(m1 >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m1, 0u))] = k1;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (c0 || c1) {
        int a0 = 0, a1 = 0;
        int x = 0;
        for (; x + 4 <= ncand; x += 4) {
            unsigned long long t[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) t[q] = cand[x + q];       // every lane reads the same key: a broadcast
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                a0 += t[q] > k0 ? 1 : 0;
                a1 += t[q] > k1 ? 1 : 0;
            }
        }
        for (; x < ncand; ++x) {
            const unsigned long long t = cand[x];
            a0 += t > k0 ? 1 : 0;
            a1 += t > k1 ? 1 : 0;
        }
        if (c0 && a0 < L) publish_u64(pkeys_slot + a0, k0);
        if (c1 && a1 < L) publish_u64(pkeys_slot + a1, k1);
    }
    if (lane < L && lane >= ncand) publish_u64(pkeys_slot + lane, kNoKey);
    __builtin_amdgcn_wave_barrier();     // the next row of this wave reuses cand
}

// The same for Q candidates per lane (tiles of more than 128 rows); `cap` keys fit `cand`.  Returns false,
// having published nothing, when more than `cap` candidates reach the threshold.
constexpr int kLargeTileCandCap = 256;
template <int Q>
__device__ __forceinline__ bool wave_publish_top_by_threshold_q(const unsigned (&ord)[Q], const int (&id)[Q], int L,
                                                                unsigned long long *cand, int cap,
                                                                unsigned long long *__restrict__ pkeys_slot,
                                                                int lane) {
    unsigned top = ord[0];
#pragma unroll
    for (int q = 1; q < Q; ++q) top = ord[q] > top ? ord[q] : top;
    unsigned T;
    if (L <= 8) {
        int gsteps = 6;
        while ((kWave >> gsteps) < L) --gsteps;
        T = wave_min_of_group_max_u32(top, gsteps);
    } else {
        T = wave_kth_largest_prefix16(top, L);
    }
    T = T == 0u ? 1u : T;
    int ncand = 0;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const bool c = ord[q] >= T;
        const unsigned long long mask = __ballot(c);
        if (mask != 0ull) {
            const int slot = ncand + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                                    __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
            if (c && slot < cap) cand[slot] = ((unsigned long long)ord[q] << 32) | (unsigned)(~(unsigned)id[q]);
            ncand += __popcll(mask);
        }
    }
    if (ncand > cap) return false;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int c = lane; c < ncand; c += kWave) {
        const unsigned long long key = cand[c];
        int above = 0;
        int x = 0;
        for (; x + 8 <= ncand; x += 8) {
            unsigned long long t[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) t[q] = cand[x + q];
#pragma unroll
            for (int q = 0; q < 8; ++q) above += t[q] > key ? 1 : 0;
        }
        for (; x < ncand; ++x) above += cand[x] > key ? 1 : 0;
        if (above < L) publish_u64(pkeys_slot + above, key);
    }
    if (lane < L && lane >= ncand) publish_u64(pkeys_slot + lane, kNoKey);
    __builtin_amdgcn_wave_barrier();     // the next row of this wave reuses cand
    return true;
}

// ------------------------------------------------------------------ workgroup epilogue of one hidden row
// zrow: the row's logit tile in LDS (S partial sums per logit, `sstride` floats
// apart).  Publishes (max, sum-exp) and the L best keys of this workgroup.
// QMAX*64 >= rows_b.  idq: target ids of tile rows lane + 64*q.
template <int QMAX>
__device__ __forceinline__ void block_epilogue_core(const float *zrow, int S, int sstride, int rows_b, int L,
                                                    const int (&idq)[QMAX], float *__restrict__ logp_full_row,
                                                    unsigned long long *__restrict__ pms_slot,
                                                    unsigned long long *__restrict__ pkeys_slot, int lane,
                                                    unsigned long long *cand = nullptr) {
    unsigned ord[QMAX];
    int id[QMAX];
    float zq[QMAX];
    float lmax = -INFINITY;
#pragma unroll
    for (int q = 0; q < QMAX; ++q) {
        const int t = lane + q * kWave;
        ord[q] = 0u;
        id[q] = idq[q];
        zq[q] = -INFINITY;
        if (t < rows_b) {
            float z = 0.f;
            for (int s = 0; s < S; ++s) z += zrow[(size_t)s * sstride + t];
            if (logp_full_row) logp_full_row[t] = z;
            zq[q] = z;
            ord[q] = orderable_f32(z);
            lmax = fmaxf(lmax, z);
        }
    }
    const float M = wave_max(lmax);
    float ls = 0.f;
#pragma unroll
    for (int q = 0; q < QMAX; ++q) ls += __expf(zq[q] - M);   // exp(-inf) = 0 for absent rows
    const float Ssum = wave_sum(ls);
    bool published = false;
    if constexpr (QMAX == 2) {
        if (cand != nullptr && L >= 5) {       // up to four rounds are no slower than the threshold (measured)
            wave_publish_top_by_threshold(ord, id, L, cand, pkeys_slot, lane);
            published = true;
        }
    } else {
        if (cand != nullptr && L >= 3 && L <= kWave)
            published = wave_publish_top_by_threshold_q<QMAX>(ord, id, L, cand, kLargeTileCandCap, pkeys_slot, lane);
    }
    if (!published) {
        const unsigned long long key = wave_select_top<QMAX>(ord, id, L, lane);
        if (lane < L) publish_u64(pkeys_slot + lane, key);
    }
    if (lane == 0)
        publish_u64(pms_slot, ((unsigned long long)__float_as_uint(Ssum) << 32) | __float_as_uint(M));
}

// small tiles (<= 128 rows): ids were prefetched by the caller
__device__ __forceinline__ void block_epilogue_small(const float *zrow, int S, int sstride, int rows_b, int L, int id0,
                                                  int id1, float *__restrict__ logp_full_row,
                                                  unsigned long long *__restrict__ pms_slot,
                                                  unsigned long long *__restrict__ pkeys_slot, int lane,
                                                  unsigned long long *cand = nullptr) {
    const int idq[2] = {id0, id1};
    block_epilogue_core<2>(zrow, S, sstride, rows_b, L, idq, logp_full_row, pms_slot, pkeys_slot, lane, cand);
}

// large tiles (<= 1024 rows): ids are read here; QMAX logits per lane, sized to the tile (4, 8 or 16)
template <int QMAX>
__device__ __forceinline__ void block_epilogue_large_q(const float *zrow, int S, int sstride, int rows_b, int L,
                                                       const int *__restrict__ map_tile,
                                                       float *__restrict__ logp_full_row,
                                                       unsigned long long *__restrict__ pms_slot,
                                                       unsigned long long *__restrict__ pkeys_slot, int lane,
                                                       unsigned long long *cand) {
    int idq[QMAX];
#pragma unroll
    for (int q = 0; q < QMAX; ++q) idq[q] = map_tile[min(lane + q * kWave, rows_b - 1)];
    block_epilogue_core<QMAX>(zrow, S, sstride, rows_b, L, idq, logp_full_row, pms_slot, pkeys_slot, lane, cand);
}
__device__ __forceinline__ void block_epilogue_large(const float *zrow, int S, int sstride, int rows_b, int L,
                                                  const int *__restrict__ map_tile,
                                                  float *__restrict__ logp_full_row,
                                                  unsigned long long *__restrict__ pms_slot,
                                                  unsigned long long *__restrict__ pkeys_slot, int lane,
                                                  unsigned long long *cand = nullptr) {
    if (rows_b <= 4 * kWave)
        block_epilogue_large_q<4>(zrow, S, sstride, rows_b, L, map_tile, logp_full_row, pms_slot, pkeys_slot, lane, cand);
    else if (rows_b <= 8 * kWave)
        block_epilogue_large_q<8>(zrow, S, sstride, rows_b, L, map_tile, logp_full_row, pms_slot, pkeys_slot, lane, cand);
    else
        block_epilogue_large_q<kStepMaxRowsPerBlock / kWave>(zrow, S, sstride, rows_b, L, map_tile, logp_full_row,
                                                             pms_slot, pkeys_slot, lane, cand);
}

// ------------------------------------------------------------------ four hidden rows per pass
// Tiles of at most 16 Q logits per hidden row (Q = 8: 128 rows, Q = 9: 144) and L <= 16: the 16 lanes of DPP row g
// rank hidden row i0 + g (Q logits per lane), so a wave finishes four hidden rows in
// the time of one.  zt: logit tile [hidden row][tp]; idq: ids of tile rows gl + 16 q.
template <int Q, bool GUARDED = false>
__device__ __forceinline__ void block_epilogue_rows4(const float *zt, int tp, int i0, int n, int rows_b, int L,
                                                     const int (&idq)[Q], float *__restrict__ logp_full, size_t k,
                                                     int row0, unsigned long long *__restrict__ pms,
                                                     unsigned long long *__restrict__ pkeys, int nlists, int blk,
                                                     int lane, unsigned long long *cand) {
    const int g = lane >> 4, gl = lane & 15;
    const int i = i0 + g;
    const bool active = i < n;
    const float *zrow = zt + (size_t)(active ? i : 0) * tp;
    unsigned ord[Q];
    int id[Q];
    float zq[Q];
    float lmax = -INFINITY;
    if constexpr (GUARDED) {
        // (a branch per logit: fewer registers live at once -- the many-row kernel has none to spare)
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int t = gl + 16 * q;
            ord[q] = 0u;
            id[q] = idq[q];
            zq[q] = -INFINITY;
            if (active && t < rows_b) {
                const float z = zrow[t];
                if (logp_full) logp_full[(size_t)i * k + row0 + t] = z;
                zq[q] = z;
                ord[q] = orderable_f32(z);
                lmax = fmaxf(lmax, z);
            }
        }
    } else {
        // every lane reads -- past the tile's end its last logit again -- and selects afterwards: no branch per logit
        // (a third of the instructions of a pass were those branches)
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int t = gl + 16 * q;
            const bool ok = active && t < rows_b;
            const float z = zrow[min(t, rows_b - 1)];
            id[q] = idq[q];
            zq[q] = ok ? z : -INFINITY;
            ord[q] = ok ? orderable_f32(z) : 0u;
            lmax = fmaxf(lmax, zq[q]);
        }
        if (logp_full != nullptr) {
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int t = gl + 16 * q;
                if (active && t < rows_b) logp_full[(size_t)i * k + row0 + t] = zq[q];
            }
        }
    }
    const float M = __uint_as_float(row16_allreduce_u32(__float_as_uint(lmax), OpMaxF32{}));
    float ls = 0.f;
#pragma unroll
    for (int q = 0; q < Q; ++q) ls += __expf(zq[q] - M);
    const float Ssum = __uint_as_float(row16_allreduce_u32(__float_as_uint(ls), OpAddF32{}));
    if (active && gl == 0)
        publish_u64(pms + (size_t)i * nlists + blk,
                    ((unsigned long long)__float_as_uint(Ssum) << 32) | __float_as_uint(M));
    if (L <= 8) {
        // Selection by threshold: T = the L-th largest of the 16 lanes' best logits, so at least L logits reach
        // it and the L best of the row are among those that do -- about L + 2 of the 128.  They are compacted
        // into 16 keys of LDS per row and each finds its rank by counting: no L dependent rounds.  More than 16
        // candidates in any row of the wave (many equal logits; 3 in 1000 rows otherwise): the rounds below.
        unsigned bo = ord[0];
#pragma unroll
        for (int q = 1; q < Q; ++q) bo = ord[q] > bo ? ord[q] : bo;
        const int above = row16_count_greater(bo);      // lanes of the row with a strictly better best logit
        // the smallest best logit that fewer than L others beat is the L-th largest
        unsigned T = row16_allreduce_u32(above < L ? bo : 0xFFFFFFFFu, OpMinU32{});
        T = T == 0u ? 1u : T;   // fewer than L lanes have logits at all: every logit is a candidate
        int cnt = 0;
#pragma unroll
        for (int q = 0; q < Q; ++q) cnt += ord[q] >= T ? 1 : 0;
        unsigned incl = (unsigned)cnt;
        incl += dpp_mov<0x111>(incl);       // row_shr:1 (lanes without a source read 0)
        incl += dpp_mov<0x112>(incl);       // row_shr:2
        incl += dpp_mov<0x114>(incl);       // row_shr:4
        incl += dpp_mov<0x118>(incl);       // row_shr:8
        const int total = (int)row16_allreduce_u32(incl, OpMaxU32{});
        if (__ballot(total > 16) == 0ull) {
            unsigned long long *crow = cand + 16 * g;
            crow[gl] = kNoKey;              // below every candidate: unused slots count for nothing
            int pos = (int)incl - cnt;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if (ord[q] >= T) crow[pos++] = ((unsigned long long)ord[q] << 32) | (unsigned)(~(unsigned)id[q]);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const unsigned long long mine = crow[gl];
            int rank = 0;
#pragma unroll
            for (int x = 0; x < 16; ++x) rank += crow[x] > mine ? 1 : 0;
            if (active) {
                unsigned long long *slot = pkeys + ((size_t)i * nlists + blk) * L;
                if (gl < total && rank < L) publish_u64(slot + rank, mine);
                if (gl < L && gl >= total) publish_u64(slot + gl, kNoKey);
            }
            __builtin_amdgcn_wave_barrier();     // the wave's next rows reuse cand
            return;
        }
    }
    unsigned res_ord = 0u, res_id = 0u;
    for (int r = 0; r < L; ++r) {
        unsigned bo = ord[0];
#pragma unroll
        for (int q = 1; q < Q; ++q) bo = ord[q] > bo ? ord[q] : bo;
        const unsigned wmax = row16_allreduce_u32(bo, OpMaxU32{});
        unsigned myid = 0xFFFFFFFFu;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (ord[q] == wmax) myid = (unsigned)id[q] < myid ? (unsigned)id[q] : myid;
        }
        const unsigned wid = row16_allreduce_u32(myid, OpMinU32{});
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (ord[q] == wmax && (unsigned)id[q] == wid) ord[q] = 0u;
        }
        if (gl == r) {
            res_ord = wmax;
            res_id = wid;
        }
    }
    if (active) {
        const unsigned long long key =
            res_ord == 0u ? kNoKey : (((unsigned long long)res_ord << 32) | (unsigned)(~res_id));
        if (gl < L) publish_u64(pkeys + ((size_t)i * nlists + blk) * L + gl, key);
    }
}

// A row's results are written through to memory (relaxed agent-scope stores, like the partials): a tree level
// fused behind the merge reads them from another workgroup, possibly on another XCD, whose L2 would not see a
// line that is still dirty in this one's.
__device__ __forceinline__ void store_result(int *__restrict__ ids_row, float *__restrict__ logp_row, int slot, int id,
                                             float logp) {
    __hip_atomic_store(ids_row + slot, id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(reinterpret_cast<unsigned *>(logp_row) + slot, __float_as_uint(logp), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// ------------------------------------------------------------------ direct merge of at most 2048 keys (one wave)
// Butterfly over the wave whose first `gsteps` steps take the maximum (inside groups of 2^gsteps
// lanes) and whose remaining steps take the minimum over those groups: the smallest group maximum.
__device__ __forceinline__ unsigned wave_min_of_group_max_u32(unsigned v, int gsteps) {
    unsigned t = dpp_mov<0xB1>(v);      // quad_perm [1,0,3,2]
    v = gsteps > 0 ? (v > t ? v : t) : (v < t ? v : t);
    t = dpp_mov<0x4E>(v);               // quad_perm [2,3,0,1]
    v = gsteps > 1 ? (v > t ? v : t) : (v < t ? v : t);
    t = dpp_mov<0x141>(v);              // row_half_mirror
    v = gsteps > 2 ? (v > t ? v : t) : (v < t ? v : t);
    t = dpp_mov<0x140>(v);              // row_mirror
    v = gsteps > 3 ? (v > t ? v : t) : (v < t ? v : t);
    auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = gsteps > 4 ? (r[0] > r[1] ? r[0] : r[1]) : (r[0] < r[1] ? r[0] : r[1]);
    r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return gsteps > 5 ? (r[0] > r[1] ? r[0] : r[1]) : (r[0] < r[1] ? r[0] : r[1]);
}

constexpr int kDirectKeysPerLane = 48;      // up to 3072 keys stay in registers (256 lists of 12)
constexpr int kDirectMaxCand = 128;

// 16 bytes per lane with the coherence of acquire_u64 (agent scope: not served from this XCD's L2).
// Issue cost per wave is that of an 8-byte load, so two keys per load halve the request time.
__device__ __forceinline__ void acquire_load16(u32x4 &dst, const void *p) {
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void wait_loads16(u32x4 (&r)[16]) {
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7]),
                   "+v"(r[8]), "+v"(r[9]), "+v"(r[10]), "+v"(r[11]), "+v"(r[12]), "+v"(r[13]), "+v"(r[14]),
                   "+v"(r[15]));
}
__device__ __forceinline__ void wait_loads24(u32x4 (&r)[24]) {
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7]),
                   "+v"(r[8]), "+v"(r[9]), "+v"(r[10]), "+v"(r[11]), "+v"(r[12]), "+v"(r[13]), "+v"(r[14]),
                   "+v"(r[15]), "+v"(r[16]), "+v"(r[17]), "+v"(r[18]), "+v"(r[19]), "+v"(r[20]), "+v"(r[21]),
                   "+v"(r[22]), "+v"(r[23]));
}

// The first active lane's value in every lane.  The row's log-sum-exp goes through this before it is subtracted
// from the logits: the lanes' copies of a wave-wide float sum can differ in the last bits (the summand is a product,
// and the compiler contracts it with the first exchange step into a fused multiply-add -- a lane's own product
// unrounded, its partner's rounded), and tokens with bit-identical logits must get bit-identical log-probs
// whichever lane writes them.
__device__ __forceinline__ float lane_uniform(float x) {
    return __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(x)));
}

// All `total` <= 64 U published keys of a hidden row (any order) are held in registers, U per lane
// (U = 32 or 48: read as U / 2 pairs, `total` even and src 16-byte aligned; U = 4: one key per load).
// With G = the power of two >= m, the lanes form G groups; every group's best logit is a different
// key, so at least G >= m keys reach T = the smallest of the group maxima, and the m best keys are
// among the keys whose logit reaches T (a few dozen).  Those are compacted into LDS and ranked by
// counting.  Returns false, having written nothing, when more than kDirectMaxCand keys reach T
// (massive ties): the caller then merges the sorted lists round by round.
// lse_fn() is called once, after the wait for the keys, and returns the row's log-sum-exp (what it reduces was
// requested by the caller before this call, so those loads and the keys' travel together); lse_out receives it.
template <int U, bool FULL, typename LseFn>
__device__ __forceinline__ bool finalize_row_direct(const unsigned long long *__restrict__ src, int total, int m,
                                                    LseFn &&lse_fn, float &lse_out, unsigned long long *stage,
                                                    int *__restrict__ out_ids_row, float *__restrict__ out_logp_row,
                                                    int lane) {
    static_assert(U == 48 || U == 32 || U == 4, "unsupported register budget");
    unsigned long long kreg[U];
    if constexpr (U >= 32) {
        u32x4 r[U / 2];
        const int npairs = total >> 1;
        // Straight-line code from the first request to the wait: the compiler does not know that these
        // registers are still in flight, and a branch in between (say, around the requests past the end)
        // makes it copy them at the join -- before their values have arrived.  Requests past the end
        // re-read the last pair instead.
#pragma unroll
        for (int u = 0; u < U / 2; ++u) {
            const int e = u * kWave + lane;
            acquire_load16(r[u], src + 2 * (FULL ? e : min(e, npairs - 1)));
        }
        if constexpr (U == 32) wait_loads16(r);
        else wait_loads24(r);
#pragma unroll
        for (int u = 0; u < U / 2; ++u) {
            const bool valid = FULL || u * kWave + lane < npairs;
            kreg[2 * u] = valid ? (((unsigned long long)r[u][1] << 32) | r[u][0]) : kNoKey;
            kreg[2 * u + 1] = valid ? (((unsigned long long)r[u][3] << 32) | r[u][2]) : kNoKey;
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) kreg[u] = acquire_u64(src + min(u * kWave + lane, total - 1));
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (u * kWave + lane >= total) kreg[u] = kNoKey;
        }
    }
    const float lse = lse_fn();
    lse_out = lse;
    unsigned top = 0u;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const unsigned o = (unsigned)(kreg[u] >> 32);
        top = o > top ? o : top;
    }
    unsigned T;
    if (m <= 8) {
        int gsteps = 6;                 // G = 64 >> gsteps groups, G >= m
        while ((kWave >> gsteps) < m) --gsteps;
        T = wave_min_of_group_max_u32(top, gsteps);
    } else {
        // 9 or more tokens: the power of two above m would make 16 or more groups and several times m candidates.
        // Instead T = the upper 16 bits of the m-th largest of the lanes' best logits, found bit by bit with ballots
        // (at least m lanes, hence m keys, reach it; if fewer than m lanes hold a key at all, T comes out as 0).
        T = wave_kth_largest_prefix16(top, m);
    }
    T = T == 0u ? 1u : T;               // an empty group: every real key is a candidate (real keys have a non-zero high word)
    int ncand = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const bool c = (unsigned)(kreg[u] >> 32) >= T;
        const unsigned long long mask = __ballot(c);
        if (mask != 0ull) {
            const int slot = ncand + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                                    __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
            if (c && slot < kDirectMaxCand) stage[slot] = kreg[u];
            ncand += __popcll(mask);
        }
    }
    if (ncand > kDirectMaxCand) return false;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int c = lane; c < ncand; c += kWave) {
        const unsigned long long key = stage[c];
        int above = 0;
        int x = 0;
        for (; x + 8 <= ncand; x += 8) {
            unsigned long long t[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) t[q] = stage[x + q];      // every lane reads the same key: a broadcast
#pragma unroll
            for (int q = 0; q < 8; ++q) above += t[q] > key ? 1 : 0;
        }
        for (; x < ncand; ++x) above += stage[x] > key ? 1 : 0;
        if (above < m) {
            store_result(out_ids_row, out_logp_row, (int)above, key_id(key), key_logit(key) - lse);
        }
    }
    __builtin_amdgcn_wave_barrier();
    return true;
}

// ------------------------------------------------------------------ final merge of one hidden row (one wave)
// pms_row: [B] (max | sumexp << 32); pkeys_row: [B][L] keys, each list sorted
// descending.  stage: wave-private LDS for (min(B, 256) + 1) * L keys.
// Lists are merged 256 at a time (4 per lane); with CARRY the best m of one
// group are carried into the next as one more list, so B is unbounded.
template <bool CARRY>
__device__ __forceinline__ void finalize_row(const unsigned long long *__restrict__ pms_row,
                                             const unsigned long long *__restrict__ pkeys_row, int B, int L, int m,
                                             unsigned long long *stage, int *__restrict__ out_ids_row,
                                             float *__restrict__ out_logp_row, float *__restrict__ out_lse_i,
                                             float *__restrict__ lse_buf_i, int lane) {
    constexpr int GROUP = kStepMaxBlocks;        // lists merged per pass
    constexpr int BQ = GROUP / kWave + (CARRY ? 1 : 0);   // lists per lane
    constexpr int U = 32;                        // 64-lane loads in flight per batch (16 KiB)
    // log-sum-exp over all lists.  Up to GROUP lists the (max, sum) words are requested first and reduced only
    // after the keys of the direct merge have been requested too: one trip to memory instead of two in a row.
    const int total_keys = B * L;
    const bool direct = m <= kWave && (total_keys <= 4 * kWave ||
                                       (total_keys <= kDirectKeysPerLane * kWave && (total_keys & 1) == 0));
    float lse;
    if (direct && B <= GROUP) {
        unsigned long long ms[GROUP / kWave];
#pragma unroll
        for (int q = 0; q < GROUP / kWave; ++q) ms[q] = acquire_u64(pms_row + min(lane + kWave * q, B - 1));
        auto lse_fn = [&]() {
            float lm = -INFINITY, ls = 0.f;
#pragma unroll
            for (int q = 0; q < GROUP / kWave; ++q) {
                if (lane + kWave * q < B) {
                    const float Mb = __uint_as_float((unsigned)ms[q]);
                    const float Sb = __uint_as_float((unsigned)(ms[q] >> 32));
                    const float Mn = fmaxf(lm, Mb);
                    ls = ls * __expf(lm - Mn) + Sb * __expf(Mb - Mn);   // exp(-inf) = 0 on the first term
                    lm = Mn;
                }
            }
            const float M = wave_max(lm);
            return lane_uniform(M + __logf(wave_sum(ls * __expf(lm - M))));
        };
        bool done;
        if (total_keys == 32 * kWave)
            done = finalize_row_direct<32, true>(pkeys_row, total_keys, m, lse_fn, lse, stage, out_ids_row, out_logp_row, lane);
        else if (total_keys > 32 * kWave)
            done = finalize_row_direct<48, false>(pkeys_row, total_keys, m, lse_fn, lse, stage, out_ids_row, out_logp_row, lane);
        else if (total_keys > 4 * kWave)
            done = finalize_row_direct<32, false>(pkeys_row, total_keys, m, lse_fn, lse, stage, out_ids_row, out_logp_row, lane);
        else
            done = finalize_row_direct<4, false>(pkeys_row, total_keys, m, lse_fn, lse, stage, out_ids_row, out_logp_row, lane);
        if (done) {
            if (lane == 0) {
                *lse_buf_i = lse;
                if (out_lse_i) *out_lse_i = lse;
            }
            return;
        }
    } else {
        float lm = -INFINITY, ls = 0.f;
        unsigned long long ms[GROUP / kWave];
        for (int b0 = 0; b0 < B; b0 += GROUP) {
#pragma unroll
            for (int q = 0; q < GROUP / kWave; ++q) ms[q] = acquire_u64(pms_row + min(b0 + lane + kWave * q, B - 1));
#pragma unroll
            for (int q = 0; q < GROUP / kWave; ++q) {
                if (b0 + lane + kWave * q < B) {
                    const float Mb = __uint_as_float((unsigned)ms[q]);
                    const float Sb = __uint_as_float((unsigned)(ms[q] >> 32));
                    const float Mn = fmaxf(lm, Mb);
                    ls = ls * __expf(lm - Mn) + Sb * __expf(Mb - Mn);   // exp(-inf) = 0 on the first term
                    lm = Mn;
                }
            }
        }
        const float M = wave_max(lm);
        lse = lane_uniform(M + __logf(wave_sum(ls * __expf(lm - M))));
    }

    unsigned res_ord = 0u;
    unsigned res_id = 0u;
    for (int b0 = 0; b0 < B; b0 += GROUP) {
        const int Bc = min(GROUP, B - b0);
        const int total = Bc * L;
        const unsigned long long *src = pkeys_row + (size_t)b0 * L;
        // everything this pass needs is requested before the first wait
        for (int base = 0; base < total; base += U * kWave) {
            unsigned long long kreg[U];
            if (base + U * kWave <= total) {
#pragma unroll
                for (int u = 0; u < U; ++u) kreg[u] = acquire_u64(src + base + u * kWave + lane);
#pragma unroll
                for (int u = 0; u < U; ++u) stage[base + u * kWave + lane] = kreg[u];
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (base + u * kWave < total) kreg[u] = acquire_u64(src + min(base + u * kWave + lane, total - 1));
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int e = base + u * kWave + lane;
                    if (e < total) stage[e] = kreg[u];
                }
            }
        }
        if constexpr (CARRY) {
            // the previous pass's result (lane r holds rank r) joins as list number Bc
            if (lane < L)
                stage[total + lane] = (b0 > 0 && lane < m && res_ord != 0u)
                                          ? (((unsigned long long)res_ord << 32) | (unsigned)(~res_id))
                                          : kNoKey;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // m rounds over the heads of the sorted lists
        const int nl = Bc + (CARRY ? 1 : 0);
        unsigned ord[BQ];
        int id[BQ];
        int pos[BQ];
#pragma unroll
        for (int q = 0; q < BQ; ++q) {
            const int b = lane + kWave * q;
            const unsigned long long key = b < nl ? stage[(size_t)b * L] : kNoKey;
            ord[q] = (unsigned)(key >> 32);
            id[q] = key_id(key);
            pos[q] = 0;
        }
        res_ord = 0u;
        res_id = 0u;
        for (int r = 0; r < m; ++r) {
            // the successor of every head is read now, so that a pop below costs no LDS round trip
            unsigned long long succ[BQ];
#pragma unroll
            for (int q = 0; q < BQ; ++q)
                succ[q] = stage[(size_t)min(lane + kWave * q, nl - 1) * L + min(pos[q] + 1, L - 1)];
            unsigned bo = ord[0];
#pragma unroll
            for (int q = 1; q < BQ; ++q) bo = ord[q] > bo ? ord[q] : bo;
            const unsigned wmax = wave_max_u32(bo);
            unsigned myid = 0xFFFFFFFFu;
            int cnt = 0;
#pragma unroll
            for (int q = 0; q < BQ; ++q) {
                if (ord[q] == wmax) {
                    myid = (unsigned)id[q] < myid ? (unsigned)id[q] : myid;
                    ++cnt;
                }
            }
            const unsigned long long holders = __ballot(cnt > 0);
            const unsigned long long multi = __ballot(cnt > 1);
            unsigned wid;
            if (__popcll(holders) == 1 && multi == 0ull) {
                wid = __builtin_amdgcn_readlane(myid, __ffsll((long long)holders) - 1);
            } else {
                wid = wave_min_u32(myid);
            }
#pragma unroll
            for (int q = 0; q < BQ; ++q) {
                const bool win = ord[q] == wmax && (unsigned)id[q] == wid && wmax != 0u;
                const unsigned long long key = pos[q] + 1 < L ? succ[q] : kNoKey;
                ord[q] = win ? (unsigned)(key >> 32) : ord[q];
                id[q] = win ? key_id(key) : id[q];
                pos[q] += win ? 1 : 0;
            }
            if (lane == r) {
                res_ord = wmax;
                res_id = wid;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    if (lane < m) {
        store_result(out_ids_row, out_logp_row, lane, (int)res_id, from_orderable_f32(res_ord) - lse);
    }
    if (lane == 0) {
        *lse_buf_i = lse;
        if (out_lse_i) *out_lse_i = lse;
    }
}

}  // namespace vt
