// Eq. 1 of the paper: V_trim = V[Top-K(c, k)], W_trim = W[Top-K(c, k), :].
//
// Selection = radix select of the k-th largest count, most significant byte first (threshold T
// and the number r of T-valued ids to keep; ties go to the lower id), then an id-ordered
// compaction that emits the selected ids already ascending -- no sort.  All of it runs over the
// whole device, one workgroup per 1024 ids, as a fixed sequence of small launches:
//   sel_zero, sel_init   digit totals of all eight byte positions of the counts
//   sel_hist (p = 6..0)  histogram of byte p among the ids whose higher bytes equal the prefix chosen
//                        so far; a byte position on which all counts agree needs none (with 10^7
//                        calibration tokens two of the seven launches do work, the others return at
//                        once), and the highest position that varies uses the totals as they are
//   sel_count, sel_write per-workgroup numbers of ids above / at the threshold, then the compaction
// No launch depends on host knowledge of the data: every workgroup re-derives the prefix, the
// remaining k and finally (T, r) from the histograms written by the launches before it.
// gather_rows_kernel: W_trim[j, :] = W[map[j], :], a pure copy at HBM speed.
#include "vt_build.h"
#include "vt_device.h"

namespace vt {

namespace {
constexpr int kSelWaves = kSelectThreads / kWave;   // 16
constexpr int kDigits = 256;
constexpr int kBytes = 8;

struct SelBufs {
    unsigned *gtot;    // [kBytes][kDigits] digit totals over all ids
    unsigned *chist;   // [kBytes][kDigits] digit totals among the ids that match the prefix above that byte
    unsigned *tab;     // [nblk][2] ids above / at the threshold per workgroup
};

// Several heads per launch (grid.y = head): head y selects k[y] of the counts at counts + y V into map[y], with
// the scratch of a single selection at scratch + y stride.
struct SelBatch {
    unsigned char *scratch;
    size_t stride;
    int nblk;
    int k[kSelectMaxHeads];
    int *map[kSelectMaxHeads];
};
__device__ __forceinline__ SelBufs head_bufs(const SelBatch &sb) {
    SelBufs b;
    b.gtot = reinterpret_cast<unsigned *>(sb.scratch + (size_t)blockIdx.y * sb.stride);
    b.chist = b.gtot + kBytes * kDigits;
    b.tab = b.chist + kBytes * kDigits;
    return b;
}

// Every kernel first copies both histogram tables (16 KiB, contiguous in the scratch) into LDS: the walk
// below reads them a few words at a time with each read depending on the previous choice.
__device__ __forceinline__ void stage_tables(const SelBufs &b, unsigned *hs) {
    for (int i = threadIdx.x; i < 2 * kBytes * kDigits; i += kSelectThreads) hs[i] = b.gtot[i];
    __syncthreads();
}

// true iff every count has the same byte p (one bin holds all V); *digit is then that byte.  All 64 lanes must call.
__device__ __forceinline__ bool byte_idle(const unsigned *__restrict__ gtot, int p, int V, int *digit = nullptr) {
    int mine = -1;
    for (int d = lane_id(); d < kDigits; d += kWave) {
        if (gtot[p * kDigits + d] == (unsigned)V) mine = d;
    }
    const unsigned long long who = __ballot(mine >= 0);
    if (who == 0ull) return false;
    if (digit != nullptr) *digit = __builtin_amdgcn_readlane(mine, __ffsll((long long)who) - 1);
    return true;
}

// Walks the byte positions from 7 down to `stop + 1`, choosing at each the digit in which the k-th
// largest count lies.  Returns the chosen bytes as `prefix` (aligned at bit 8 * (stop + 1)) and the
// number `krem` of ids still to take among those that match the prefix; `top` = highest byte position
// on which the counts differ (-1 if none).  All 64 lanes of the calling wave take part and get the
// same result.
struct SelState {
    unsigned long long prefix;
    int krem;
    int top;
};
__device__ __forceinline__ SelState sel_state(const unsigned *hs, int V, int k, int stop) {
    const unsigned *gtot = hs, *chist = hs + kBytes * kDigits;
    const int lane = lane_id();
    SelState s;
    s.prefix = 0ull;
    s.krem = k;
    s.top = -1;
    for (int q = kBytes - 1; q > stop; --q) {
        int same = 0;
        const bool idle = byte_idle(gtot, q, V, &same);
        if (idle) {      // nothing to choose at this position, and nobody to leave behind
            s.prefix = (s.prefix << 8) | (unsigned long long)same;
            continue;
        }
        if (s.top < 0) s.top = q;
        const unsigned *H = q == s.top ? gtot + q * kDigits : chist + q * kDigits;
        // lane l holds digits 255 - 4 l .. 252 - 4 l (descending); inclusive scan over lanes
        unsigned v[4], sum = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[i] = H[255 - (4 * lane + i)];
            sum += v[i];
        }
        unsigned inc = sum;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const unsigned t = __shfl_up(inc, o);
            if (lane >= o) inc += t;
        }
        const unsigned long long hit = __ballot(inc >= (unsigned)s.krem);
        // hit is never empty: the candidates number at least krem
        const int first = __ffsll((long long)hit) - 1;
        unsigned above = inc - sum;        // ids in higher digits, as seen by this lane
        int dsel = 0;
        unsigned asel = 0;
        bool found = false;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (!found && above + v[i] >= (unsigned)s.krem) {
                dsel = 255 - (4 * lane + i);
                asel = above;
                found = true;
            }
            above += v[i];
        }
        const int d = __builtin_amdgcn_readlane(dsel, first);
        const unsigned a = (unsigned)__builtin_amdgcn_readlane((int)asel, first);
        s.prefix = (s.prefix << 8) | (unsigned long long)d;
        s.krem -= (int)a;
    }
    return s;
}

__global__ void __launch_bounds__(256) sel_zero_kernel(SelBatch sb, int nwords) {
    unsigned *p = head_bufs(sb).gtot;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < nwords; i += gridDim.x * 256) p[i] = 0u;
}

__global__ void __launch_bounds__(kSelectThreads) sel_init_kernel(const long long *__restrict__ counts_all, int V,
                                                                  SelBatch sb) {
    const SelBufs b = head_bufs(sb);
    const long long *__restrict__ counts = counts_all + (size_t)blockIdx.y * V;
    __shared__ unsigned h[kBytes * kDigits];
    for (int i = threadIdx.x; i < kBytes * kDigits; i += kSelectThreads) h[i] = 0u;
    __syncthreads();
    const int j = blockIdx.x * kSelectThreads + threadIdx.x;
    const bool in = j < V;
    const unsigned long long c = in ? (unsigned long long)counts[j] : 0ull;
    const unsigned long long live = __ballot(in);
    // the upper bytes are the same in nearly every count (zero): when a whole wave agrees on a digit one
    // lane adds for all, instead of 64 LDS atomics queueing on one address
#pragma unroll
    for (int p = 0; p < kBytes; ++p) {
        const int dg = (int)((c >> (8 * p)) & 255ull);
        const int first = __builtin_amdgcn_readfirstlane(dg);
        const unsigned long long same = __ballot(in && dg == first);
        if (same == live && live != 0ull) {
            if (lane_id() == __ffsll((long long)live) - 1) atomicAdd(&h[p * kDigits + dg], (unsigned)__popcll(live));
        } else if (in) {
            atomicAdd(&h[p * kDigits + dg], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kBytes * kDigits; i += kSelectThreads) {
        if (h[i] != 0u) atomicAdd(&b.gtot[i], h[i]);
    }
}

__global__ void __launch_bounds__(kSelectThreads) sel_hist_kernel(const long long *__restrict__ counts_all, int V,
                                                                  int p, SelBatch sb) {
    const SelBufs b = head_bufs(sb);
    const long long *__restrict__ counts = counts_all + (size_t)blockIdx.y * V;
    const int k = sb.k[blockIdx.y];
    __shared__ unsigned h[kDigits];
    __shared__ unsigned hs[2 * kBytes * kDigits];
    // this thread's count is requested first: it depends on nothing, and its trip to memory passes while the
    // tables are staged and walked (these kernels are chains of latencies, not of work)
    const int j = blockIdx.x * kSelectThreads + threadIdx.x;
    const unsigned long long c = j < V ? (unsigned long long)counts[j] : 0ull;
    stage_tables(b, hs);
    if (byte_idle(hs, p, V)) return;
    const SelState s = sel_state(hs, V, k, p);
    if (s.top < 0 || p >= s.top) return;          // the highest varying byte uses the totals themselves
    if (threadIdx.x < kDigits) h[threadIdx.x] = 0u;
    __syncthreads();
    if (j < V) {
        if ((c >> (8 * (p + 1))) == s.prefix) atomicAdd(&h[(int)((c >> (8 * p)) & 255ull)], 1u);
    }
    __syncthreads();
    if (threadIdx.x < kDigits && h[threadIdx.x] != 0u) atomicAdd(&b.chist[p * kDigits + threadIdx.x], h[threadIdx.x]);
}

// T = the k-th largest count, r = how many ids with count == T are kept (the lowest ids)
__device__ __forceinline__ void sel_threshold(const unsigned *hs, int V, int k, unsigned long long &T, int &r) {
    const SelState s = sel_state(hs, V, k, -1);
    T = s.prefix;
    r = s.krem;
}

__global__ void __launch_bounds__(kSelectThreads) sel_count_kernel(const long long *__restrict__ counts_all, int V,
                                                                   SelBatch sb) {
    const SelBufs b = head_bufs(sb);
    const long long *__restrict__ counts = counts_all + (size_t)blockIdx.y * V;
    const int k = sb.k[blockIdx.y];
    __shared__ int s_gt[kSelWaves], s_eq[kSelWaves];
    __shared__ unsigned hs[2 * kBytes * kDigits];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int j = blockIdx.x * kSelectThreads + tid;
    const unsigned long long c = j < V ? (unsigned long long)counts[j] : 0ull;      // requested before the walk
    stage_tables(b, hs);
    unsigned long long T;
    int r;
    sel_threshold(hs, V, k, T, r);
    const int ngt = __popcll(__ballot(j < V && c > T)), neq = __popcll(__ballot(j < V && c == T));
    if (lane == 0) {
        s_gt[w] = ngt;
        s_eq[w] = neq;
    }
    __syncthreads();
    if (tid == 0) {
        int g = 0, e = 0;
        for (int q = 0; q < kSelWaves; ++q) {
            g += s_gt[q];
            e += s_eq[q];
        }
        b.tab[2 * blockIdx.x] = (unsigned)g;
        b.tab[2 * blockIdx.x + 1] = (unsigned)e;
    }
}

__global__ void __launch_bounds__(kSelectThreads) sel_write_kernel(const long long *__restrict__ counts_all, int V,
                                                                   SelBatch sb) {
    const SelBufs b = head_bufs(sb);
    const long long *__restrict__ counts = counts_all + (size_t)blockIdx.y * V;
    const int k = sb.k[blockIdx.y];
    int *__restrict__ map = sb.map[blockIdx.y];
    __shared__ int s_gt[kSelWaves + 1], s_eq[kSelWaves + 1];
    __shared__ int s_red[2 * kSelWaves];
    __shared__ unsigned hs[2 * kBytes * kDigits];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    // requested before the walk: this thread's count, and the ids above / at the threshold in the workgroups
    // before this one
    const int j = blockIdx.x * kSelectThreads + tid;
    const unsigned long long c = j < V ? (unsigned long long)counts[j] : 0ull;
    int gb = 0, eb = 0;
    for (int x = tid; x < (int)blockIdx.x; x += kSelectThreads) {
        gb += (int)b.tab[2 * x];
        eb += (int)b.tab[2 * x + 1];
    }
    stage_tables(b, hs);
    unsigned long long T;
    int r;
    sel_threshold(hs, V, k, T, r);
    gb = wave_sum_i32(gb);
    eb = wave_sum_i32(eb);
    if (lane == 0) {
        s_red[w] = gb;
        s_red[kSelWaves + w] = eb;
    }
    const bool gt = j < V && c > T, eq = j < V && c == T;
    const unsigned long long bg = __ballot(gt), be = __ballot(eq);
    if (lane == 0) {
        s_gt[w + 1] = __popcll(bg);
        s_eq[w + 1] = __popcll(be);
    }
    __syncthreads();
    if (tid == 0) {
        int g = 0, e = 0;
        for (int q = 0; q < kSelWaves; ++q) {
            g += s_red[q];
            e += s_red[kSelWaves + q];
        }
        s_gt[0] = g;
        s_eq[0] = e;
        for (int q = 1; q <= kSelWaves; ++q) {
            s_gt[q] += s_gt[q - 1];
            s_eq[q] += s_eq[q - 1];
        }
    }
    __syncthreads();
    const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    const int gt_before = s_gt[w] + __popcll(bg & below);
    const int eq_before = s_eq[w] + __popcll(be & below);
    if (gt || (eq && eq_before < r)) map[gt_before + min(eq_before, r)] = j;
}

}  // namespace

size_t select_scratch_bytes(int V) {
    const size_t nblk = ((size_t)V + kSelectThreads - 1) / kSelectThreads;
    return (2 * kBytes * kDigits + 2 * nblk) * sizeof(unsigned);
}

size_t select_scratch_stride(int V) { return (select_scratch_bytes(V) + 255) / 256 * 256; }

// counts: [n_heads, V]; scratch: n_heads * select_scratch_stride(V) bytes
void launch_select_topk_heads(const long long *counts, int V, int n_heads, const int *k, void *scratch, int *const *map,
                              hipStream_t st) {
    SelBatch sb;
    sb.scratch = static_cast<unsigned char *>(scratch);
    sb.stride = select_scratch_stride(V);
    sb.nblk = (V + kSelectThreads - 1) / kSelectThreads;
    for (int hd = 0; hd < kSelectMaxHeads; ++hd) {
        sb.k[hd] = hd < n_heads ? k[hd] : 1;
        sb.map[hd] = hd < n_heads ? map[hd] : nullptr;
    }
    const dim3 grid(sb.nblk, n_heads);
    hipLaunchKernelGGL(sel_zero_kernel, dim3(4, n_heads), dim3(256), 0, st, sb, 2 * kBytes * kDigits);
    hipLaunchKernelGGL(sel_init_kernel, grid, dim3(kSelectThreads), 0, st, counts, V, sb);
    for (int p = kBytes - 2; p >= 0; --p)
        hipLaunchKernelGGL(sel_hist_kernel, grid, dim3(kSelectThreads), 0, st, counts, V, p, sb);
    hipLaunchKernelGGL(sel_count_kernel, grid, dim3(kSelectThreads), 0, st, counts, V, sb);
    hipLaunchKernelGGL(sel_write_kernel, grid, dim3(kSelectThreads), 0, st, counts, V, sb);
}

void launch_select_topk(const long long *counts, int V, int k, void *scratch, int *map, hipStream_t st) {
    launch_select_topk_heads(counts, V, 1, &k, scratch, &map, st);
}

// One wave copies one row at a time with 16-byte lanes, four loads in flight; rows are independent.
__device__ __forceinline__ void copy_row(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t nvec, int lane) {
    size_t c = lane;
    for (; c + 3 * kWave < nvec; c += 4 * kWave) {
        const u32x4 a0 = __builtin_nontemporal_load(src + c);
        const u32x4 a1 = __builtin_nontemporal_load(src + c + kWave);
        const u32x4 a2 = __builtin_nontemporal_load(src + c + 2 * kWave);
        const u32x4 a3 = __builtin_nontemporal_load(src + c + 3 * kWave);
        __builtin_nontemporal_store(a0, dst + c);
        __builtin_nontemporal_store(a1, dst + c + kWave);
        __builtin_nontemporal_store(a2, dst + c + 2 * kWave);
        __builtin_nontemporal_store(a3, dst + c + 3 * kWave);
    }
    for (; c < nvec; c += kWave) __builtin_nontemporal_store(__builtin_nontemporal_load(src + c), dst + c);
}

__global__ void __launch_bounds__(256) gather_rows_kernel(const char *__restrict__ W, size_t row_bytes,
                                                          const int *__restrict__ map, int k,
                                                          char *__restrict__ W_trim) {
    const int lane = lane_id();
    const int wave = (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    const int nwaves = (int)((gridDim.x * blockDim.x) >> 6);
    const size_t nvec = row_bytes >> 4;
    for (int j = wave; j < k; j += nwaves) {
        copy_row(reinterpret_cast<const u32x4 *>(W + (size_t)map[j] * row_bytes),
                 reinterpret_cast<u32x4 *>(W_trim + (size_t)j * row_bytes), nvec, lane);
    }
}

// The same for several heads in one launch (grid.y = head).
struct GatherBatch {
    int k[kSelectMaxHeads];
    const int *map[kSelectMaxHeads];
    char *W_trim[kSelectMaxHeads];
};
__global__ void __launch_bounds__(256) gather_rows_heads_kernel(const char *__restrict__ W, size_t row_bytes,
                                                                GatherBatch gb) {
    const int lane = lane_id();
    const int wave = (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    const int nwaves = (int)((gridDim.x * blockDim.x) >> 6);
    const size_t nvec = row_bytes >> 4;
    const int k = gb.k[blockIdx.y];
    const int *__restrict__ map = gb.map[blockIdx.y];
    char *__restrict__ W_trim = gb.W_trim[blockIdx.y];
    for (int j = wave; j < k; j += nwaves) {
        copy_row(reinterpret_cast<const u32x4 *>(W + (size_t)map[j] * row_bytes),
                 reinterpret_cast<u32x4 *>(W_trim + (size_t)j * row_bytes), nvec, lane);
    }
}

void launch_gather_rows_heads(const void *W, size_t row_bytes, int n_heads, const int *k, const int *const *map,
                              void *const *W_trim, hipStream_t st) {
    GatherBatch gb;
    int kmax = 1;
    for (int hd = 0; hd < kSelectMaxHeads; ++hd) {
        gb.k[hd] = hd < n_heads ? k[hd] : 0;
        gb.map[hd] = hd < n_heads ? map[hd] : nullptr;
        gb.W_trim[hd] = hd < n_heads ? static_cast<char *>(W_trim[hd]) : nullptr;
        if (hd < n_heads && k[hd] > kmax) kmax = k[hd];
    }
    int blocks = (kmax + 3) / 4;          // 4 waves per workgroup
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(gather_rows_heads_kernel, dim3(blocks, n_heads), dim3(256), 0, st, static_cast<const char *>(W),
                       row_bytes, gb);
}

void launch_gather_rows(const void *W, size_t row_bytes, const int *map, int k, void *W_trim, hipStream_t st) {
    int blocks = (k + 3) / 4;          // 4 waves per workgroup
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const char *>(W), row_bytes,
                       map, k, static_cast<char *>(W_trim));
}

}  // namespace vt
