// Internal interface of the draft-tree selection kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace vt {

constexpr int kTreeThreads = 1024;
constexpr int kTreeCountMaxN = 1024;    // up to here every candidate's rank is found by counting
constexpr int kTreeMaxN = 16384;        // above: a bitonic sort of the keys in LDS (128 KiB at the limit)
constexpr int kTreeMaxKeepSorted = 1024;   // index-ordered output: at most this many kept nodes

struct TreeArgs {
    const float *parent_cum;   // [n] or null (rerank: scores are taken as they are)
    const float *vals;         // [N] step log-probs (expansion) or cumulative scores (rerank)
    const int *ids;            // [N] or null
    int N, m, K;
    int index_order;           // 0: best first; 1: ascending candidate index
    int *out_a;                // expansion: parent [K]; rerank: node index [K]
    int *out_token;            // [K] or null
    float *out_score;          // [K] or null
};

hipError_t launch_tree_select(const TreeArgs &a, hipStream_t st);

}  // namespace vt
