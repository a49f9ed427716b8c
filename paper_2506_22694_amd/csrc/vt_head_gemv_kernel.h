// Draft step for a few hidden rows (n <= 8): bandwidth-bound GEMV-class kernel.
//
// Algorithm 2's drafting lines with a trimmed head: z = h W_trim^T over the k
// trimmed rows, then log-softmax over those k logits, the m best per hidden row
// and the map back to target ids.
//
// Data flow of one workgroup (8 waves):
//   * it owns `rpb` consecutive rows of W_trim;
//   * a wave streams whole rows (or one of S column segments of them): each
//     load instruction fetches 64 lanes x 16 B = 1 KiB contiguous, non-temporal,
//     with several rows in flight per wave (a hand-written load pipeline);
//   * h lives in registers (packed bf16, or fp32), a lane owning the same
//     columns of every row, so the stream is consumed by dot2 / fma only;
//   * after a batch of 4 or 8 rows a "transposed" wave reduction (permlane swaps + DPP) leaves
//     one finished logit per lane, which goes to an LDS tile;
//   * the workgroup epilogue turns the tile into (max, sum-exp) and the
//     workgroup's best m candidates per hidden row;
//   * the kernel ends there; step_finalize_kernel (a workgroup per hidden row)
//     merges the partials: lse, top-m, remap.
#pragma once
#include "vt_device.h"
#include "vt_launch.h"
#include "vt_step.h"
#include "vt_step_tail.h"
#include <type_traits>

namespace vt {

// ------------------------------------------------------------------ dot
// acc + a.lo * b.lo + a.hi * b.hi on packed bf16 pairs (products exact in fp32).
// The operands are passed as plain scalars: bit-casting a vector element
// expression directly reads element 0 whatever the swizzle.
__device__ __forceinline__ float dot2_bf16(unsigned a, unsigned b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc,
                                           false);
}

template <bool BF16>
__device__ __forceinline__ float dot_chunk(const u32x4 &w, const u32x4 &x, float acc) {
    if constexpr (BF16) {
        acc = dot2_bf16(w.x, x.x, acc);
        acc = dot2_bf16(w.y, x.y, acc);
        acc = dot2_bf16(w.z, x.z, acc);
        acc = dot2_bf16(w.w, x.w, acc);
    } else {
        acc = fmaf(__uint_as_float(w.x), __uint_as_float(x.x), acc);
        acc = fmaf(__uint_as_float(w.y), __uint_as_float(x.y), acc);
        acc = fmaf(__uint_as_float(w.z), __uint_as_float(x.z), acc);
        acc = fmaf(__uint_as_float(w.w), __uint_as_float(x.w), acc);
    }
    return acc;
}

// ------------------------------------------------------------------ explicit load pipeline
// The row stream is software-pipelined by hand: the loads and their waits are
// inline assembly so that the compiler neither hoists a batch's loads into one
// cluster (which needs twice the registers) nor splits them.  vmcnt counts this
// wave's outstanding vector-memory operations, which return in issue order.
//
// 16 bytes per lane from (uniform base + per-lane byte offset), streaming hint.
__device__ __forceinline__ void stream_load16(u32x4 &dst, unsigned voff, const void *sbase) {
    asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(dst) : "v"(voff), "s"(sbase) : "memory");
}
// Wait until at most N vector-memory operations are outstanding.  The row buffer
// is passed through so that its consumers cannot be scheduled above the wait.
template <int N, int CS>
__device__ __forceinline__ void wait_row(u32x4 (&b)[CS]) {
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    if constexpr (CS == 1) {
        asm volatile("s_waitcnt vmcnt(%1)" : "+v"(b[0]) : "n"(N));
    } else if constexpr (CS == 2) {
        asm volatile("s_waitcnt vmcnt(%2)" : "+v"(b[0]), "+v"(b[1]) : "n"(N));
    } else if constexpr (CS == 3) {
        asm volatile("s_waitcnt vmcnt(%3)" : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]) : "n"(N));
    } else if constexpr (CS == 4) {
        asm volatile("s_waitcnt vmcnt(%4)" : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]) : "n"(N));
    } else {
        static_assert(CS == 6, "unsupported chunk count");
        asm volatile("s_waitcnt vmcnt(%6)"
                     : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5])
                     : "n"(N));
    }
}
// Orders what follows after the last update of a row's accumulators (an empty
// statement the scheduler cannot move accumulators or later loads across).
template <int NP>
__device__ __forceinline__ void pin_after(float (&acc)[NP]) {
    if constexpr (NP == 1) {
        asm volatile("" : "+v"(acc[0]));
    } else if constexpr (NP == 2) {
        asm volatile("" : "+v"(acc[0]), "+v"(acc[1]));
    } else if constexpr (NP == 4) {
        asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]));
    } else {
        static_assert(NP == 8, "unsupported row count");
        asm volatile(""
                     : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]),
                       "+v"(acc[6]), "+v"(acc[7]));
    }
}

// ------------------------------------------------------------------ transposed wave reduction
// Each lane holds V partial sums v[0..V).  On return v[0] of lane l is the
// 64-lane total of value number (l >> (6 - log2 V)); every total is formed by
// the same balanced tree over lanes whatever its number, so two rows of W with
// identical bits give identical logits.
template <int D>
__device__ __forceinline__ float lane_xor(float x) {
    if constexpr (D == 8) {
        return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x128 /*row_ror:8*/,
                                                           0xF, 0xF, false));
    } else if constexpr (D == 2) {
        return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x4E /*quad_perm 2,3,0,1*/,
                                                           0xF, 0xF, false));
    } else if constexpr (D == 1) {
        return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0xB1 /*quad_perm 1,0,3,2*/,
                                                           0xF, 0xF, false));
    } else {
        return __shfl_xor(x, D);
    }
}

// one stage: values a (kept by lanes with bit D clear) and b (kept by lanes with bit D set)
template <int D>
__device__ __forceinline__ float xstage(float a, float b, int lane) {
    if constexpr (D == 32) {
        auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    } else if constexpr (D == 16) {
        auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    } else {
        const bool hi = (lane & D) != 0;
        const float send = hi ? a : b;
        const float keep = hi ? b : a;
        return keep + lane_xor<D>(send);
    }
}

template <int V>
__device__ __forceinline__ float xreduce(float (&v)[V], int lane) {
    static_assert(V == 8 || V == 16 || V == 32 || V == 64, "V must be 8..64");
    // stage D=32
    constexpr int c0 = V;
#pragma unroll
    for (int j = 0; j < c0 / 2; ++j) v[j] = xstage<32>(v[j], v[j + c0 / 2], lane);
    constexpr int c1 = c0 / 2;
#pragma unroll
    for (int j = 0; j < c1 / 2; ++j) v[j] = xstage<16>(v[j], v[j + c1 / 2], lane);
    constexpr int c2 = c1 / 2;
#pragma unroll
    for (int j = 0; j < c2 / 2; ++j) v[j] = xstage<8>(v[j], v[j + c2 / 2], lane);
    constexpr int c3 = c2 / 2;   // V=8 -> 1
    if constexpr (c3 >= 2) {
#pragma unroll
        for (int j = 0; j < c3 / 2; ++j) v[j] = xstage<4>(v[j], v[j + c3 / 2], lane);
    } else {
        v[0] += lane_xor<4>(v[0]);
    }
    constexpr int c4 = c3 >= 2 ? c3 / 2 : 1;
    if constexpr (c4 >= 2) {
#pragma unroll
        for (int j = 0; j < c4 / 2; ++j) v[j] = xstage<2>(v[j], v[j + c4 / 2], lane);
    } else {
        v[0] += lane_xor<2>(v[0]);
    }
    constexpr int c5 = c4 >= 2 ? c4 / 2 : 1;
    if constexpr (c5 >= 2) {
        v[0] = xstage<1>(v[0], v[1], lane);
    } else {
        v[0] += lane_xor<1>(v[0]);
    }
    return v[0];
}

// ------------------------------------------------------------------ the kernel
// Rows per reduction batch (R) and row buffers in flight per wave (NSLOT, a
// power of two dividing R), chosen so that h registers + accumulators + row
// buffers stay below 256 VGPRs (two waves per SIMD).
template <int NP>
struct BatchRows {
    static constexpr int value = NP >= 8 ? 4 : 8;
};
template <int NP, int CS>
struct SlotsFor {
    static constexpr int R = BatchRows<NP>::value;
    static constexpr int room = (216 - 4 * CS * NP - R * NP) / (4 * CS);
    static constexpr int cap = room < R ? room : R;
    static constexpr int value = cap >= 8 ? 8 : (cap >= 4 ? 4 : 2);
};

template <bool BF16, int NP, int CS>
__global__ void __launch_bounds__(kStepWaves *kWave) head_gemv_kernel(const StepArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *zt = reinterpret_cast<float *>(smem);
    constexpr int NW = kStepWaves;
    constexpr int EPC = BF16 ? 8 : 4;   // elements per 16-byte chunk
    constexpr int ES = BF16 ? 2 : 4;    // element size
    constexpr int R = BatchRows<NP>::value;   // rows per batch
    constexpr int RSH = R == 8 ? 3 : 2;
    constexpr int NSLOT = SlotsFor<NP, CS>::value;
    constexpr int V = R * NP;

    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave index, uniform
    const int S = a.S;
    const int s = w % S;   // column segment of this wave; waves with equal s share its rows
    const int row0 = blockIdx.x * a.rpb;
    const int rows_b = min(a.rpb, a.k - row0);
    const size_t rs = (size_t)a.d * ES;   // row stride in bytes

    // Columns this lane owns in every row.  A lane whose columns lie beyond d
    // streams column 0 instead (always in bounds) against zeroed h registers,
    // so the loads need no predicate.
    int coff[CS];
    bool cval[CS];
    unsigned voff[CS];
#pragma unroll
    for (int c = 0; c < CS; ++c) {
        const int col = ((s * CS + c) * kWave + lane) * EPC;
        cval[c] = col < a.d;
        coff[c] = cval[c] ? col * ES : 0;
        voff[c] = (unsigned)coff[c];
    }

    // A wave keeps NSLOT rows in flight.  Past the end of the tile it streams h
    // instead (resident in L2, always in bounds): no branch around any load, so
    // the load counter stays exact.
    const char *Wb = static_cast<const char *>(a.W) + (size_t)row0 * rs;
    auto load_row = [&](int row, u32x4(&dst)[CS]) {
        const char *p = row < rows_b ? Wb + (size_t)row * rs : static_cast<const char *>(a.h);
#pragma unroll
        for (int c = 0; c < CS; ++c) stream_load16(dst[c], voff[c], p);
    };
    u32x4 wb[NSLOT][CS];
    int rowq[R];   // rows of the batch being reduced (uniform values)
#pragma unroll
    for (int x = 0; x < NSLOT; ++x) {
        rowq[x] = (w / S) * NSLOT + x;
        load_row(rowq[x], wb[x]);      // the longest latency of the kernel starts first
    }
#pragma unroll
    for (int x = NSLOT; x < R; ++x) rowq[x] = rows_b;   // filled as the batch proceeds

    // hidden rows -> registers (zeros where the column or the row does not exist)
    u32x4 hreg[CS][NP];
#pragma unroll
    for (int c = 0; c < CS; ++c) {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int ii = (int)((a.row_pack >> (8 * min(i, a.n - 1))) & 0xFFull);
            hreg[c][i] = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(a.h) + (size_t)ii * rs + coff[c]);
        }
    }
    if (a.ticket_clear != nullptr && blockIdx.x == 0 && threadIdx.x == 0)
        __hip_atomic_store(a.ticket_clear, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // target ids of the tile rows this lane will rank in the epilogue (small tiles)
    const int id0 = a.map[row0 + min(lane, rows_b - 1)];
    const int id1 = a.map[row0 + min(lane + kWave, rows_b - 1)];
#pragma unroll
    for (int c = 0; c < CS; ++c) {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const unsigned keep = (cval[c] && i < a.n) ? 0xFFFFFFFFu : 0u;
            hreg[c][i].x &= keep;
            hreg[c][i].y &= keep;
            hreg[c][i].z &= keep;
            hreg[c][i].w &= keep;
        }
    }

    // Rows are dealt to the waves of a segment team round-robin.  (Handing them out
    // dynamically from an LDS counter balances the two waves of a SIMD, the older
    // of which runs ahead, but measured slower overall.)
    const int G = NW / S;
    int next_row = G * NSLOT + w / S;
    auto take_row = [&]() -> int {
        const int v = next_row;
        next_row += G;
        return v;
    };

    while (rowq[0] < rows_b) {
        float acc[R][NP];
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int i = 0; i < NP; ++i) acc[r][i] = 0.f;
        }
        int nextq[NSLOT];   // rows that will occupy the slots after this batch's refills
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int slot = r % NSLOT;
            const int fresh = take_row();
            // the slot's loads are the oldest outstanding: everything but the younger slots must be back
            wait_row<CS *(NSLOT - 1), CS>(wb[slot]);
#pragma unroll
            for (int c = 0; c < CS; ++c) {
#pragma unroll
                for (int i = 0; i < NP; ++i) acc[r][i] = dot_chunk<BF16>(wb[slot][c], hreg[c][i], acc[r][i]);
            }
            pin_after<NP>(acc[r]);
            load_row(fresh, wb[slot]);
            if (r + NSLOT < R) rowq[r + NSLOT] = fresh;   // later row of this batch
            else nextq[(r + NSLOT) - R] = fresh;          // row of the next batch
        }
        float flat[V];
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int i = 0; i < NP; ++i) flat[r * NP + i] = acc[r][i];
        }
        const float tot = xreduce<V>(flat, lane);
        // lane l holds value number (l >> (6 - log2 V)) = r * NP + i
        constexpr int SH = V == 64 ? 0 : (V == 32 ? 1 : (V == 16 ? 2 : 3));
        static_assert(V >= 8, "at least 8 values per batch");
        {
            const int idx = lane >> SH;
            const int r = idx / NP, i = idx % NP;
            int t = rowq[0];
#pragma unroll
            for (int q = 1; q < R; ++q) t = r == q ? rowq[q] : t;
            if ((lane & ((1 << SH) - 1)) == 0 && t < rows_b) zt[(size_t)(s * NP + i) * a.tpitch + t] = tot;
        }
#pragma unroll
        for (int x = 0; x < NSLOT; ++x) rowq[x] = nextq[x];
#pragma unroll
        for (int x = NSLOT; x < R; ++x) rowq[x] = rows_b;
    }
    // loads past the end of the tile are still in flight: let them land before their registers are reused
#pragma unroll
    for (int x = 0; x < NSLOT; ++x) wait_row<0, CS>(wb[x]);
    __syncthreads();

    if (a.zbuf != nullptr) {
        // store-only tail (many tokens per row): the tile's logits, summed over the column segments, go to
        // z [n, k]; a workgroup per hidden row finishes the step (row_select_kernel)
        const int sstride = NP * a.tpitch;
        for (int i = w; i < a.n; i += NW) {
            for (int t = lane; t < rows_b; t += kWave) {
                float v = 0.f;
                for (int s2 = 0; s2 < S; ++s2) v += zt[(size_t)s2 * sstride + (size_t)i * a.tpitch + t];
                a.zbuf[(size_t)i * a.k + row0 + t] = v;
            }
        }
        return;
    }

    {
        const int sstride = NP * a.tpitch;
        for (int i = w; i < a.n; i += NW) {
            const float *zrow = zt + (size_t)i * a.tpitch;
            float *full = a.out_logp_full ? a.out_logp_full + (size_t)i * a.k + row0 : nullptr;
            unsigned long long *pms_slot = a.pms + (size_t)i * a.nblocks + blockIdx.x;
            unsigned long long *pk_slot = a.pkeys + ((size_t)i * a.nblocks + blockIdx.x) * a.L;
            // candidate keys of the threshold selection sit behind the tile: kLargeTileCandCap per wave
            unsigned long long *cand = reinterpret_cast<unsigned long long *>(
                                           smem + (((size_t)S * sstride * sizeof(float) + 15) & ~(size_t)15)) +
                                       (size_t)w * kLargeTileCandCap;
            if (rows_b <= 2 * kWave)
                block_epilogue_small(zrow, S, sstride, rows_b, a.L, id0, id1, full, pms_slot, pk_slot, lane, cand);
            else
                block_epilogue_large(zrow, S, sstride, rows_b, a.L, a.map + row0, full, pms_slot, pk_slot, lane, cand);
        }
    }
}

template <bool BF16, int NP, int CS>
inline hipError_t launch_gemv_inst(const StepArgs &a, size_t lds, hipStream_t st) {
    auto kern = head_gemv_kernel<BF16, NP, CS>;
    // allow large dynamic LDS (the logit tile of tall row blocks), once per device
    static LdsLimitOnce lds_limit;
    hipError_t e = allow_dynamic_lds(lds_limit, {reinterpret_cast<const void *>(kern)}, kMaxDynamicLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(a.nblocks), dim3(kStepWaves * kWave), lds, st, a);
    return hipGetLastError();
}

}  // namespace vt
