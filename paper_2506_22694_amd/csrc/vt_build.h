// Internal interface of the calibration-side kernels (count, select, gather).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace vt {

// ---- Algorithm 1 ----
constexpr int kHistBinsPerBlock = 65536;   // 16-bit bins privatised in LDS per workgroup (128 KiB, two per word)
constexpr int kHistBlocks = 256;           // workgroups per launch: id-stream chunks x bin ranges
constexpr int kHistThreads = 1024;
constexpr int kHistUnroll = 6;            // 16-byte id vectors in flight per thread (4 / 6 / 8: 28.2 / 28.0 / 28.8 us at
                                          // 10^7 ids, 141.8 / 137.8 / 135.7 us at 10^8)

int hist_num_ranges(int V);
int hist_num_chunks(int64_t n_ids, int V);
// partial: [chunks, V rounded up to even] 16-bit scratch
hipError_t launch_count_tokens(const void *ids, bool ids64, int64_t n_ids, int V, long long *counts,
                         unsigned long long *n_invalid, unsigned *partial, hipStream_t st);

// ---- Eq. 1 ----
constexpr int kSelectThreads = 1024;
constexpr int kSelectMaxHeads = 16;        // heads per batched launch (VT_MAX_HEADS)
// scratch: select_scratch_bytes(V) of device memory, no initialisation
size_t select_scratch_bytes(int V);
void launch_select_topk(const long long *counts, int V, int k, void *scratch, int *map, hipStream_t st);
void launch_gather_rows(const void *W, size_t row_bytes, const int *map, int k, void *W_trim, hipStream_t st);
// several heads per launch sequence (grid.y = head): counts [n_heads, V]; scratch n_heads * select_scratch_stride(V)
size_t select_scratch_stride(int V);
void launch_select_topk_heads(const long long *counts, int V, int n_heads, const int *k, void *scratch, int *const *map,
                              hipStream_t st);
void launch_gather_rows_heads(const void *W, size_t row_bytes, int n_heads, const int *k, const int *const *map,
                              void *const *W_trim, hipStream_t st);

// ---- Sec. 3.2: frequency-rank order, Top-P / minimum-count choice of k ----
constexpr int kRankSortThreads = 1024;
size_t rank_sort_scratch_bytes(int n);
// sorts all n ids by (count desc, id asc); out_ids [n_ids] receives the first n_ids of them, out_counts [n] (or
// null) all sorted counts
void launch_rank_sort(const long long *counts, int n, void *scratch, int *out_ids, int n_ids, long long *out_counts,
                      hipStream_t st);
// out: [3] = k, mass of the k largest counts, total mass; scratch: choose_k_scratch_bytes(V)
size_t choose_k_scratch_bytes(int V);
void launch_choose_k(const long long *sorted_counts, int V, int mode, double P, long long f_min, void *scratch,
                     long long *out, hipStream_t st);

}  // namespace vt
