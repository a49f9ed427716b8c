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

// ---- wave-wide reductions (all 64 lanes receive the result) ----
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        unsigned long long t = __shfl_xor(v, o);
        v = t > v ? t : v;
    }
    return v;
}
__device__ __forceinline__ int wave_sum_i32(int v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Per (block, hidden row) partial result of the draft step, merged by the
// finalize stage:  running maximum M, sum of exp(z - M), and the block's best
// candidates as keys sorted descending.
struct StepPartials {
    float *pmax;                 // [B, n]
    float *psum;                 // [B, n]
    unsigned long long *pkeys;   // [B, n, L]
    int L;                       // candidates kept per (block, row) = min(m, rows per block)
};

}  // namespace vt
