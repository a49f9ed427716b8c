// Device-side helpers shared by the vocabtrim HIP kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vt {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63u); }

// ---- total order on (logit desc, target id asc) packed into one 64-bit key ----
// Larger key == better candidate: larger logit first, then the lower target id.
// -0.0 is folded into +0.0 first so that equal logits compare equal.
__device__ __forceinline__ unsigned orderable_f32(float z) {
    if (z == 0.0f) z = 0.0f;
    unsigned u = __float_as_uint(z);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_orderable_f32(unsigned o) {
    unsigned u = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
    return __uint_as_float(u);
}
__device__ __forceinline__ unsigned long long make_key(float z, int id) {
    return ((unsigned long long)orderable_f32(z) << 32) | (unsigned)(~(unsigned)id);
}
__device__ __forceinline__ float key_logit(unsigned long long key) {
    return from_orderable_f32((unsigned)(key >> 32));
}
__device__ __forceinline__ int key_id(unsigned long long key) { return (int)(~(unsigned)key); }
// key 0 is below every real candidate (a real key has a non-zero high word unless
// the logit is a negative NaN; NaN inputs are outside the contract).
constexpr unsigned long long kNoKey = 0ull;

// ---- wave-wide all-reductions on DPP / permlane swaps (no LDS traffic) ----
// Four DPP steps reduce within a row of 16 lanes; permlane16_swap and
// permlane32_swap (gfx950) then combine the four rows.  Every lane receives the
// result and the combination order is fixed, so float sums are reproducible from run to run.
// (Lane to lane a float sum may differ in the last bits when the summand is a product: the compiler
// may contract it with the first step into a fused multiply-add.  Where all lanes must use the same
// value, take one lane's.)
template <int CTRL>
__device__ __forceinline__ unsigned dpp_mov(unsigned v) {
    return __builtin_amdgcn_update_dpp(0u, v, CTRL, 0xF, 0xF, false);
}
template <typename Op>
__device__ __forceinline__ unsigned wave_allreduce_u32(unsigned v, Op op) {
    v = op(v, dpp_mov<0xB1>(v));    // quad_perm [1,0,3,2]
    v = op(v, dpp_mov<0x4E>(v));    // quad_perm [2,3,0,1]
    v = op(v, dpp_mov<0x141>(v));   // row_half_mirror
    v = op(v, dpp_mov<0x140>(v));   // row_mirror
    auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = op(r[0], r[1]);
    r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return op(r[0], r[1]);
}
// Same, restricted to the 16 lanes of a DPP row (four independent groups per wave).
template <typename Op>
__device__ __forceinline__ unsigned row16_allreduce_u32(unsigned v, Op op) {
    v = op(v, dpp_mov<0xB1>(v));    // quad_perm [1,0,3,2]
    v = op(v, dpp_mov<0x4E>(v));    // quad_perm [2,3,0,1]
    v = op(v, dpp_mov<0x141>(v));   // row_half_mirror
    return op(v, dpp_mov<0x140>(v));   // row_mirror
}
// Lane i of a 16-lane row receives v of lane (i - S) mod 16 of the same row (row_ror:S), 1 <= S <= 15.
template <int S>
__device__ __forceinline__ unsigned row16_rotate_by(unsigned v) {
    return __builtin_amdgcn_update_dpp(0u, v, 0x120 + S, 0xF, 0xF, false);
}
// Number of the other 15 lanes of the row whose v is strictly greater than this lane's.
template <int S = 15>
__device__ __forceinline__ int row16_count_greater(unsigned v) {
    if constexpr (S == 0) {
        return 0;
    } else {
        return (row16_rotate_by<S>(v) > v ? 1 : 0) + row16_count_greater<S - 1>(v);
    }
}
struct OpMaxU32 {
    __device__ __forceinline__ unsigned operator()(unsigned a, unsigned b) const { return a > b ? a : b; }
};
struct OpMinU32 {
    __device__ __forceinline__ unsigned operator()(unsigned a, unsigned b) const { return a < b ? a : b; }
};
struct OpAddU32 {
    __device__ __forceinline__ unsigned operator()(unsigned a, unsigned b) const { return a + b; }
};
struct OpMaxF32 {
    __device__ __forceinline__ unsigned operator()(unsigned a, unsigned b) const {
        return __float_as_uint(fmaxf(__uint_as_float(a), __uint_as_float(b)));
    }
};
struct OpAddF32 {
    __device__ __forceinline__ unsigned operator()(unsigned a, unsigned b) const {
        return __float_as_uint(__uint_as_float(a) + __uint_as_float(b));
    }
};
__device__ __forceinline__ unsigned wave_max_u32(unsigned v) { return wave_allreduce_u32(v, OpMaxU32{}); }
__device__ __forceinline__ unsigned wave_min_u32(unsigned v) { return wave_allreduce_u32(v, OpMinU32{}); }
__device__ __forceinline__ float wave_max(float v) {
    return __uint_as_float(wave_allreduce_u32(__float_as_uint(v), OpMaxF32{}));
}
__device__ __forceinline__ float wave_sum(float v) {
    return __uint_as_float(wave_allreduce_u32(__float_as_uint(v), OpAddF32{}));
}
__device__ __forceinline__ int wave_sum_i32(int v) { return (int)wave_allreduce_u32((unsigned)v, OpAddU32{}); }
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        unsigned long long t = __shfl_xor(v, o);
        v = t > v ? t : v;
    }
    return v;
}

// ---- cross-workgroup publication without cache-wide fences ----
// Partials are written with relaxed agent-scope atomic stores (write-through past
// the XCD-local L2) and read back with relaxed agent-scope atomic loads (which
// do not hit in the reader's L2).  A device-scope release fence would instead
// write back the whole L2 -- tens of microseconds on this part.
__device__ __forceinline__ void publish_u64(unsigned long long *p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long acquire_u64(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Wait until every store this wave has issued is acknowledged (vmcnt(0)).
__device__ __forceinline__ void wait_stores_done() { __builtin_amdgcn_s_waitcnt(0x0F70); }

}  // namespace vt
