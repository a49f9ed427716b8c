// Internal interface between the draft-step host code and its kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace vt {

// Limits shared by host sizing code and kernels.
constexpr int kStepWaves = 8;          // waves per workgroup of the draft-step kernels
constexpr int kStepMaxBlocks = 256;    // one workgroup per CU on MI355X
constexpr int kStepMaxRowsPerBlock = 1024;
constexpr int kStepMaxK = kStepMaxBlocks * kStepMaxRowsPerBlock;
constexpr int kFinalizeLdsBytes = 152 * 1024;  // staging budget of the finalize stage
constexpr int kMaxDynamicLds = 159 * 1024;     // dynamic LDS the step kernels may request (160 KiB per CU less static use)
constexpr int kTicketBytes = 2048;             // head of a step workspace: the ticket word of a fused tree level
constexpr int kGemvMaxN = 8;           // the VALU GEMV path covers n <= 8
// The small-n kernel ends after publishing its lists and a separate merge kernel (a workgroup per hidden row)
// follows.  Merging in the kernel's last workgroup to arrive (arrival counters, no second launch) was the first
// design; it lost from 4 hidden rows on at once, and at every n since the merge kernel waits for memory once
// (k = 65536, d = 3072: n = 1 64.9 against 66.3 us, n = 2 67.8 / 69.3; k = 128256: n = 1 119.3 / 120.8, n = 3
// 123.5 / 124.9; d = 2048: 82.9 / 84.2): the counters cost more than the kernel boundary.
// ... but from 2 hidden rows on the matrix-core kernel is faster (n = 2: 38.7 against 39.4 us, n = 3: 38.8 / 39.9) when its 128-row tiles fill the 256 CUs in
// one round (measured at d = 3072, n = 8: k = 28672: 36.9 against 37.4 us, 30720: 38.7 / 40.8, 32768: 39.9 / 41.8;
// k = 24576: a tie; k = 16384: 29.8 / 27.4, k = 65536: 78.0 / 75.1)
// (d = 8192, n = 8: 97.8 against 88.0 us: only up to d = 4096, where 2048, 3072 and 4096 all gain)
constexpr int kMfmaSmallMaxD = 4096;
// wider heads gain from five rows on (n = 8: d = 5120: 61.1 / 58.0 us, 7168: 81.3 / 78.0; n = 2..4: a tie), d = 8192
// does not (87.4 / 92.8)
constexpr int kMfmaSmallMaxDManyRows = 7168;
constexpr int kMfmaSmallManyRows = 5;
// a single hidden row gains up to d = 3072 (d = 2048: 27.9 against 28.6 us, d = 3072: 36.0 / 36.4) and loses at
// d = 4096 (45.6 / 45.1)
constexpr int kMfmaSmallMaxDOneRow = 3072;
// (re-measured with all of h in LDS, n = 8, small-n / matrix-core kernel: k = 26624: 37.1 / 33.7 us, 24576: 33.6 / 32.1,
// 22528: 32.3 / 30.7, 20480: 29.8 / 29.6, 16384: 26.5 / 27.9)
constexpr int kMfmaSmallMinTiles = 160;
// Smaller heads: tiles of 64 or 32 rows, the columns of a 16-row group split over 2 or 4 waves (n = 8, small-n /
// matrix-core kernel: k = 16384: 26.1 / 24.7 us, 12288: 22.9 / 21.8, 8192: 19.0 / 18.0; n = 1: k = 8192: 17.2 / 14.8;
// n = 4: 20.8 / 17.8).  Tiles of 32 rows pay from about 96 of them (k = 5000, 157 tiles: n = 8 18.1 / 16.1,
// n = 1 14.6 / 12.7; k = 3072: a tie).
constexpr int kMfmaSmallMinTiles32 = 96;

struct StepArgs {
    const void *h;            // [n, d]
    const void *W;            // [k, d]
    const int *map;           // [k]
    int n, k, d, m;
    int S;                    // number of column segments d is split into across waves
    int rpb;                  // vocabulary rows per workgroup (multiple of 8)
    int tpitch;               // pitch (floats) of one row of the LDS logit tile
    int L;                    // candidates kept per (workgroup, hidden row) = min(m, rpb)
    int nblocks;
    unsigned long long *pms;    // [n, nblocks]  max | sumexp << 32
    unsigned long long *pkeys;  // [n, nblocks, L] candidate keys, sorted descending per list
    float *out_logp_full;     // [n, k] or null (raw logits are written first, lse subtracted later)
    float *zbuf;              // [n, k] or null: store the logits and leave the rest of the step to row_select_kernel
    // hidden row i is row (row_pack >> 8 i) & 255 of h: 0x0706050403020100 for rows 0 .. n-1, other values when
    // the rows are picked out of a larger batch (several heads per call)
    unsigned long long row_pack;
    // or null: a word the kernel sets to zero (the merge kernel behind it counts its workgroups there when a tree
    // level is fused; the kernel boundary orders the two)
    unsigned *ticket_clear;
};

// ---- matrix-core path (n > 8) ----
constexpr int kMfmaTileRows = 128;     // rows of W_trim per workgroup (16 per wave)
constexpr int kRowSelectMinL = 11;      // matrix-core path: with more tokens per row than this (8 with more than 8 hidden rows), or
constexpr int kRowSelectMinLManyRows = 8;
// small-n path: the same switch when L > 12 - n / 2 (measured crossovers: L = 8 at n = 8, 10 at n = 4, 11-12 at n = 1)
constexpr int kGemvRowSelectBase = 12;
constexpr int kRowSelectMinWork = 1280; // with n * min(m, 128) from this value on, the kernel stores its logits and a
                                        // workgroup per hidden row finishes the step
constexpr int kMfmaPrefetchUnits = 3;  // 128-column units of W_trim in flight per wave; an h chunk that has a successor
                                       // is a multiple of this many units
constexpr int kMfmaChunkPieces = 9;    // an h chunk is prefetched through registers: at most this many
                                       // 16-byte pieces per thread, i.e. 16 * NT * KC * 2 <= 9 * 512 * 16 bytes

struct MfmaArgs {
    const void *h;            // [n, d] bf16
    const void *W;            // [k, d] bf16
    const int *map;           // [k]
    int n, k, d, m;
    int L;                    // candidates kept per (tile, hidden row) = min(m, 128)
    int nlists;               // number of tiles = workgroups = candidate lists per hidden row
    int KC;                   // columns of h resident in LDS at a time (multiple of 128)
    int hpitch;               // bytes per hidden row in LDS = KC * 2 + 16
    unsigned long long *pms;    // [n, nlists]
    unsigned long long *pkeys;  // [n, nlists, L]
    float *out_logp_full;     // [n, k] or null
    void *hpack;              // more than 64 hidden rows: h re-laid in operand order, d * NT * 32 bytes
    float *zbuf;              // [n, k] or null: store the logits and leave the rest of the step to row_select_kernel
    // indexed != 0 (n <= 8 only): hidden row i is row (row_pack >> 8 i) & 255 of h -- rows picked out of a
    // larger batch (several heads per call); the merge kernel maps the output rows the same way
    unsigned long long row_pack;
    int indexed;
    // 1, 2 or 4 (n <= 8, all of h in LDS, no zbuf): tiles of 16 * nwaves / ksplit rows, ksplit waves share 16 rows
    // and the columns; nlists counts those tiles
    int ksplit;
    // waves per workgroup: kStepWaves, or (n <= 8, all of h in LDS, no zbuf) any multiple of ksplit up to
    // kMfmaMaxWaves, so that the tiles can be sized to cover the head in one round of at most 256 workgroups
    int nwaves;
    // extra_rows != 0 (8 waves, no column split): the tile is 128 + extra_rows rows, 1 <= extra_rows <= 16; the rows
    // past the 128th form one more 16-row group -- up to 8 hidden rows (all of h in LDS, d a multiple of 1024) its
    // columns are shared by the eight waves; with more hidden rows their columns follow h's chunk in LDS (16 more
    // rows of hpitch bytes) and their accumulators live in 3 * NT KiB of LDS at byte offset xoff (behind the chunk,
    // clear of the logit tile of the epilogue, inside the launch's LDS)
    int extra_rows;
    int xoff;
    // or null: a word the kernel sets to zero (the merge kernel behind it counts its workgroups there when a tree
    // level is fused; the kernel boundary orders the two)
    unsigned *ticket_clear;
};

// Several heads in one launch of the matrix-core kernel (up to 8 hidden rows in all): the tiles of head i are the
// workgroups tile_first[i] .. tile_first[i + 1] - 1, each head cut into tiles of the launch's height on its own
// (the last one ragged); hidden row r belongs to head (head_of_row >> 8 r) & 255.  Every tile multiplies all hidden
// rows -- they share the 16-row operand anyway -- and publishes an empty list for the rows of other heads.
struct MultiHeadTable {
    const void *W[16];
    const int *map[16];
    int k[16];
    int tile_first[17];
    unsigned long long head_of_row;
    int n_heads;
};
struct SingleHead {};      // the kernels' second argument when there is one head

struct FinalizeArgs {
    const unsigned long long *pms;
    const unsigned long long *pkeys;
    int nlists, L, n, m;
    int conc;                 // hidden rows (waves) per workgroup
    int stage_keys;           // LDS keys reserved per wave
    int *out_ids;
    float *out_logp;
    float *out_lse;           // or null
    float *lse_buf;
    unsigned long long row_pack;   // indexed != 0 (n <= 8): hidden row i writes output row (row_pack >> 8 i) & 255
    int indexed;
    // Tree level fused behind the merge (tree_cum != null; rows in order, n * m <= kFinalizeTreeMaxN): every
    // workgroup takes a ticket after its row; the last one ranks the n * m candidates tree_cum[i] + logp[i][j]
    // and keeps the tree_K best.
    const float *tree_cum;
    int tree_K;
    int *tree_parent;
    int *tree_token;
    float *tree_score;
    unsigned *ticket;          // one word, zeroed by the kernel that produced the lists (ticket_clear); returns to zero
};
constexpr int kFinalizeTreeMaxN = 512;

constexpr int kMfmaMaxWaves = 12;      // three waves per SIMD: 168 registers each
constexpr int kMfmaFewWaves = 7;       // more than 8 hidden rows: the instantiation for 5 .. 7 waves (smaller tiles for heads that
                                       // would leave CUs idle with 128-row tiles)

size_t mfma_stage_bytes(int nwaves);

size_t mfma_wide_lds_bytes();   // NT >= 8: two shared unit buffers
hipError_t launch_head_mfma(int NT, const MfmaArgs &a, size_t lds, hipStream_t st);
// a.W, a.map, a.k are not read: the table names every head's; a.nlists = tile_first[n_heads]
hipError_t launch_head_mfma_multi(const MfmaArgs &a, const MultiHeadTable &t, size_t lds_bytes, hipStream_t st);
hipError_t launch_step_finalize(const FinalizeArgs &f, size_t lds, hipStream_t st);

// Launchers, one translation unit per padded row count NP (1, 2, 4, 8).
// hipErrorInvalidValue if (bf16, CS) is not instantiated.
hipError_t launch_head_gemv_np1(bool bf16, int CS, const StepArgs &a, size_t lds, hipStream_t st);
hipError_t launch_head_gemv_np2(bool bf16, int CS, const StepArgs &a, size_t lds, hipStream_t st);
hipError_t launch_head_gemv_np4(bool bf16, int CS, const StepArgs &a, size_t lds, hipStream_t st);
hipError_t launch_head_gemv_np8(bool bf16, int CS, const StepArgs &a, size_t lds, hipStream_t st);

// logp_full[i, j] -= lse[i]
void launch_sub_lse(float *logp_full, const float *lse, int n, int k, hipStream_t st);
// zero the arrival counters
void launch_ws_clear(unsigned *p, int nwords, hipStream_t st);
void launch_stream_read(const void *p, size_t bytes, unsigned *sink, hipStream_t st);

// Hidden rows of one head inside a multi-head step: passed to the kernels by value.
constexpr int kMultiMaxRows = 256;
struct RowList {
    int n;
    short idx[kMultiMaxRows];
};
void launch_gather_h_rows(const void *h, void *staging, size_t row_bytes, const RowList &rows, hipStream_t st);
void launch_scatter_rows(const int *ids_s, const float *logp_s, const float *lse_s, int m, int *out_ids,
                         float *out_logp, float *out_lse, const RowList &rows, hipStream_t st);
// per-row tail on stored logits z [n, k]: lse, the m best logits and their target ids (one workgroup per row)
void launch_row_select(const float *z, const int *map, int n, int k, int m, int *out_ids, float *out_logp,
                       float *out_lse, float *lse_buf, hipStream_t st);

}  // namespace vt
