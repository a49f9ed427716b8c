// C ABI of libvocabtrim.so: argument validation, workspace layout, kernel dispatch.
// Every entry point only enqueues work on the caller's stream.
#include "vocabtrim.h"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <mutex>

#include "vt_build.h"
#include "vt_step.h"
#include "vt_tree.h"

namespace {

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int elem_size(int dtype) { return dtype == VT_BF16 ? 2 : 4; }

// last HIP error seen by this thread's calls into the library (for vt_last_device_error)
thread_local hipError_t g_last_hip_error = hipSuccess;

inline int device_status(hipError_t e) {
    if (e == hipSuccess) return VT_OK;
    g_last_hip_error = e;
    return VT_ERR_DEVICE;
}
inline int launch_status() { return device_status(hipGetLastError()); }

// ---------------------------------------------------------------- library-owned step workspace
// Device memory of the draft step for callers that cannot allocate (vt_draft_head_step_static): one array per
// GPU, alive from the moment the code object is loaded on it until the process ends.  In host code the array's
// name is only a handle; the device address is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[VT_STATIC_WS_BYTES];
std::mutex g_scratch_mutex;
void *g_scratch_ptr[64] = {};      // per device ordinal; written under the mutex, never changed afterwards

int static_scratch_of_current_device(void **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return device_status(e);
    if (dev < 0 || dev >= 64) return device_status(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return device_status(e);
        if (p == nullptr) return device_status(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return VT_OK;
}

// ---------------------------------------------------------------- draft-step plan
// Workgroups one round of the draft-step kernels may have: the compute units of the current device (one workgroup
// per CU: they take most of a CU's LDS), read once per process; 256 on MI355X, which is also the most the kernels'
// tables are sized for and the answer where no device is visible (the workspace-size functions are pure host code).
// The measured crossovers below (so many tiles of so many rows) are scaled to it.
int round_workgroups() {
    static const int cus = []() {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
            (void)hipGetLastError();
            return vt::kStepMaxBlocks;
        }
        return n < vt::kStepMaxBlocks ? n : vt::kStepMaxBlocks;
    }();
    return cus;
}

struct StepPlan {
    bool ok = false;
    bool gemv = false;     // small-n VALU path
    bool mfma = false;     // matrix-core path
    int NP = 0, CS = 0, S = 0;
    int NT = 0, nlists = 0, KC = 0, hpitch = 0, fin_stage_keys = 0, ksplit = 1, nwaves = vt::kStepWaves;
    size_t fin_lds = 0;
    int rpb = 0, nblocks = 0, tpitch = 0, L = 0, fin_conc = 0;
    size_t lds = 0;
    // workspace layout (byte offsets)
    size_t off_lse = 0, off_pms = 0, off_pkeys = 0, off_hpack = 0, off_zbuf = 0, bytes = 0;
    bool row_select = false;   // matrix-core path: logits stored, one workgroup per hidden row finishes
    int extra_rows = 0;        // matrix-core path: tile rows past the 128th (shared by the eight waves, or in LDS beside h)
    int xoff = 0;              // ... more than 8 hidden rows: LDS offset of their accumulators
};

using vt::kTicketBytes;

// fixed: a tile shape the caller has chosen (several heads in one launch): waves, column split, number of tiles
struct FixedTiles {
    int nwaves = 0, ksplit = 1, nlists = 0;
};
StepPlan plan_step_impl(int n, int k, int d, int m, int dtype, bool force_gemv, const FixedTiles &fixed = FixedTiles{});
// force_gemv: the caller needs what only the small-n kernel offers (row picking, the fused tree level)
StepPlan plan_step(int n, int k, int d, int m, int dtype, bool force_gemv = false) {
    StepPlan p = plan_step_impl(n, k, d, m, dtype, force_gemv);
    if (!p.ok && !force_gemv && n <= vt::kGemvMaxN) p = plan_step_impl(n, k, d, m, dtype, true);
    return p;
}
StepPlan plan_step_impl(int n, int k, int d, int m, int dtype, bool force_gemv, const FixedTiles &fixed) {
    StepPlan p;
    if (n <= 0 || k <= 0 || d <= 0 || m <= 0 || k > vt::kStepMaxK) return p;
    const int CUS = round_workgroups();
    int rpb = (k + CUS - 1) / CUS;
    rpb = (rpb + 7) / 8 * 8;
    p.rpb = rpb;
    p.nblocks = (k + rpb - 1) / rpb;
    p.tpitch = rpb + 1;
    p.L = m < rpb ? m : rpb;
    p.fin_conc = 1;      // the merge kernel takes one hidden row per workgroup

    // Up to 8 rows on the matrix-core kernel: its tiles must fill most of the 256 CUs in exactly one round.  A
    // tile is 16 rows per group of KS waves (KS = 1, 2, 4 waves share a group's columns) and a workgroup has up to
    // kMfmaMaxWaves waves, so the tile height follows from the head: ceil(k / 256) rows rounded up to whole groups
    // (k = 32768: 8 waves x 16 rows; the paper's k ~ 33000: 9 waves, 144 rows, 229 - 244 tiles; k = 22786: 6 groups
    // of 2 waves, 96 rows, 238 tiles).  The split needs the kernel's own epilogue (few tokens per row), whole
    // 128-column units per wave and all of h in LDS at once.
    int ksplit = 0, nwaves = vt::kStepWaves, extra_rows = 0;
    if (!force_gemv && dtype == VT_BF16 && (d % 128) == 0 &&
        (d <= vt::kMfmaSmallMaxD || (n >= vt::kMfmaSmallManyRows && d <= vt::kMfmaSmallMaxDManyRows)) &&
        (n >= 2 || d <= vt::kMfmaSmallMaxDOneRow) && n <= vt::kGemvMaxN) {
        auto feasible = [&](int KS, int NW) {
            if (NW < KS || NW % KS != 0 || NW > vt::kMfmaMaxWaves) return false;
            const int tr = 16 * (NW / KS);
            const int tiles = (k + tr - 1) / tr;
            if (tiles < (KS == 4 ? vt::kMfmaSmallMinTiles32 : vt::kMfmaSmallMinTiles) * CUS / vt::kStepMaxBlocks || tiles > CUS)
                return false;
            // (the split also needs all of h in LDS at once: d <= 4096)
            if (KS > 1 && ((d / 128) % KS != 0 || m > vt::kRowSelectMinL || d > vt::kMfmaSmallMaxD)) return false;
            if (NW != vt::kStepWaves) {
                // another number of waves: all of h in LDS beside their staging buffers, fetched in one go
                if (vt::mfma_stage_bytes(NW) + 8 * ((size_t)d * 2 + 16) > (size_t)vt::kMaxDynamicLds) return false;
                if ((size_t)d > (size_t)vt::kMfmaChunkPieces * NW * 64) return false;
            }
            return true;
        };
        const int R = (k + CUS - 1) / CUS;                                    // rows per tile for one tile per CU
        const int G = (R + 15) / 16;                                          // ... in 16-row groups
        if (R > vt::kMfmaTileRows && R <= vt::kMfmaTileRows + 16 && (d % 1024) == 0 && (d % 2048) != 0 &&
            d <= vt::kMfmaSmallMaxD) {
            // 129 .. 144 rows per tile -- the paper's own trimmed sizes, k = 32959 .. 35010 -- : eight waves with 16
            // rows each and the rows past the 128th as one more group whose columns the eight waves share; the
            // tile is exactly R rows, so all 256 CUs stream equal shares (k = 32975, d = 3072: n = 8 40.1 us against
            // 41.4 with nine waves on 229 CUs and 41.8 on the small-n kernel, n = 1 37.0 / 37.4 / 38.9).  Rows a
            // multiple of 2 KiB long lose on it (d = 4096: 54.0 / 51.4 / 51.7 us, d = 2048: 30.1 / 27.5 / 29.1) and
            // take nine waves.
            ksplit = 1;
            nwaves = vt::kStepWaves;
            extra_rows = R - vt::kMfmaTileRows;
        }
        // more or fewer waves than eight where that measured faster than the choices below (n = 8, d = 3072:
        // k = 40000, ten waves: 46.4 against 47.5 us; 49152, twelve: 53.6 / 55.1; 20000, five groups of two: 29.1 / 29.7;
        // six groups of two measured slower; nine waves: see above)
        if (ksplit == 0 && G == 9 && feasible(1, G)) {
            ksplit = 1;
            nwaves = G;
        }
        if (ksplit == 0 && G >= 10 && feasible(1, G)) {
            ksplit = 1;
            nwaves = G;
        }
        // six waves of 16 rows (k = 20481 .. 24576: 214 - 256 tiles instead of 160 - 192 of 128 rows) pay for up to 4
        // hidden rows, seven for one (k = 22786, d = 3072: n = 1 27.4 against 28.2 us, n = 2 27.5 / 28.4, n = 4 30.8 /
        // 31.2, n = 8 32.2 / 31.7; d = 2048, n = 1: 20.6 / 21.9; k = 26000, n = 1: 29.9 / 30.1, n = 2: a tie)
        if (ksplit == 0 && ((G == 6 && n <= 4) || (G == 7 && n == 1)) && feasible(1, G)) {
            ksplit = 1;
            nwaves = G;
        }
        if (ksplit == 0 && G == 5 && feasible(2, 10)) {
            ksplit = 2;
            nwaves = 10;
        }
        // otherwise eight waves and the tile that fills the chip best
        for (int KS = 1; KS <= 4 && ksplit == 0; KS *= 2) {
            if (feasible(KS, vt::kStepWaves)) {
                ksplit = KS;
                nwaves = vt::kStepWaves;
            }
        }
    }
    if (fixed.nwaves != 0) {
        // (the same limits as above: whole units per wave, the kernel's own epilogue, all of h in LDS at once)
        ksplit = 0;
        nwaves = vt::kStepWaves;
        extra_rows = 0;
        if (dtype == VT_BF16 && (d % 128) == 0 && d <= vt::kMfmaSmallMaxD && n <= vt::kGemvMaxN && m <= vt::kRowSelectMinL &&
            (d / 128) % fixed.ksplit == 0 && (fixed.ksplit == 1 || fixed.nwaves == vt::kStepWaves) &&
            fixed.nwaves >= vt::kStepWaves && fixed.nwaves <= vt::kMfmaMaxWaves &&
            vt::mfma_stage_bytes(fixed.nwaves) + 8 * ((size_t)d * 2 + 16) <= (size_t)vt::kMaxDynamicLds &&
            (size_t)d <= (size_t)vt::kMfmaChunkPieces * fixed.nwaves * 64) {
            ksplit = fixed.ksplit;
            nwaves = fixed.nwaves;
        } else {
            return p;
        }
    }
    const bool prefer_mfma = ksplit != 0;
    if (n <= vt::kGemvMaxN && !prefer_mfma) {
        const int NP = n <= 1 ? 1 : (n <= 2 ? 2 : (n <= 4 ? 4 : 8));
        const int epc = dtype == VT_BF16 ? 8 : 4;
        const int CT = (d + 64 * epc - 1) / (64 * epc);
        static const int cs_bf16[] = {1, 2, 3, 4, 6};
        static const int cs_f32[] = {1, 2, 4};
        const int *cs_set = dtype == VT_BF16 ? cs_bf16 : cs_f32;
        const int ncs = dtype == VT_BF16 ? 5 : 3;
        for (int S = 1; S <= vt::kStepWaves && !p.gemv; S *= 2) {
            const int need = (CT + S - 1) / S;
            for (int q = 0; q < ncs; ++q) {
                const int CS = cs_set[q];
                if (CS >= need && CS * NP <= 24) {
                    const size_t tile = (size_t)S * NP * p.tpitch * sizeof(float);
                    if (tile <= 96 * 1024) {
                        p.gemv = true;
                        p.NP = NP;
                        p.CS = CS;
                        p.S = S;
                        // + 2 KiB per wave behind the tile: candidate keys of the epilogue's threshold selection
                        p.lds = ((tile + 15) & ~(size_t)15) + (size_t)vt::kStepWaves * 256 * sizeof(unsigned long long);
                    }
                    break;
                }
            }
        }
    }
    if (!p.gemv) {
        // larger n or d: the matrix-core path (bf16, d a multiple of 128, n <= 256)
        if (dtype != VT_BF16 || (d % 128) != 0 || n > 256) return p;
        int NT = 1;
        while (16 * NT < n) NT *= 2;
        const bool var_waves = prefer_mfma && nwaves != vt::kStepWaves;
        size_t stage = NT >= 8 ? vt::mfma_wide_lds_bytes() : vt::mfma_stage_bytes(var_waves ? nwaves : vt::kStepWaves);
        // More than 8 hidden rows and 129 .. 144 rows per tile for one tile per CU (the paper's trimmed sizes again):
        // tiles of exactly that many rows (k = 32975, n = 64, d = 4096: 258 tiles of 128 rows took 104 us, a nearly
        // empty second round).  With two groups of hidden rows (9 .. 16 rows are padded to 32) the columns of the rows
        // past the 128th sit in LDS beside h's chunk (16 more rows) and their accumulators behind it (3 KiB per
        // group); with four groups they are multiplied in a pass after the march (measured crossover: the kernel's
        // comment has the figures).
        const int Rx = (k + CUS - 1) / CUS;
        const bool xany = n > vt::kGemvMaxN && NT <= 4 && d >= 1024 && Rx > vt::kMfmaTileRows &&
                          Rx <= vt::kMfmaTileRows + 16;
        if (xany && NT == 1) NT = 2;
        // ... and fewer than 112 rows per tile for one tile per CU: tiles of 5 .. 7 waves (16 rows each) instead of
        // leaving CUs idle with 128-row tiles
        const int Gx = (Rx + 15) / 16;
        // (their threads must still prefetch a chunk of at least three units of h through their registers)
        const bool few = n > vt::kGemvMaxN && NT <= 4 && !xany && Gx >= 5 && Gx <= vt::kMfmaFewWaves &&
                         (size_t)vt::kMfmaChunkPieces * Gx * 64 * 16 >= (size_t)16 * (NT < 2 ? 2 : NT) * 2 * 128 * vt::kMfmaPrefetchUnits;
        if (few && NT == 1) NT = 2;
        const int NWx = few ? Gx : vt::kStepWaves;      // waves of a workgroup for more than 8 hidden rows
        if (few) stage = vt::mfma_stage_bytes(NWx);
        const bool xrows = xany && NT == 2;      // ... in LDS beside the chunk
        const bool xpass = xany && NT == 4;      // ... after the march
        const size_t xbytes = xrows ? (size_t)3 * NT * 1024 : 0;
        int KC = 128;   // NT >= 8: h is not staged at all (B-operands come from L2)
        if (NT < 8) {
            // up to 8 hidden rows occupy 8 rows of LDS (the other half of the 16-row operand repeats them)
            const size_t hrows = (n <= 8 ? 8 : 16 * (size_t)NT) + (xrows ? 16 : 0);
            const size_t hmax = ((size_t)vt::kMaxDynamicLds - stage - xbytes) / hrows;
            if (hmax < 272) return p;
            KC = (int)(((hmax - 16) / 2) / 128) * 128;
            int kc_regs = (int)((vt::kMfmaChunkPieces * (var_waves ? nwaves : NWx) * 64 * 16) / (hrows * 2) / 128 * 128);
            if (xrows) {
                // the extra rows' pieces start at a piece number of their own behind h's
                const int T = vt::kStepWaves * 64;
                kc_regs = (kc_regs / 128 + 1) * 128;
                do {
                    kc_regs -= 128;
                } while (kc_regs > 0 && (16 * NT * (kc_regs / 8) + T - 1) / T + (16 * (kc_regs / 8) + T - 1) / T > vt::kMfmaChunkPieces);
                if (kc_regs <= 0) return p;
            }
            if (KC > kc_regs) KC = kc_regs;   // the chunk must fit the register prefetch
            if (KC >= d) {
                KC = d;
            } else {
                // several chunks: near-equal sizes (d = 2560: 2304 + 256 -> 1536 + 1024), every chunk but the
                // last a multiple of the kernel's prefetch depth in 128-column units
                const int U = d / 128, P = vt::kMfmaPrefetchUnits;
                const int umax = KC / 128 / P * P;
                if (umax < P) return p;
                const int nch = (U + umax - 1) / umax;
                KC = (((U + nch - 1) / nch + P - 1) / P * P) * 128;
            }
        }
        p.mfma = true;
        p.NT = NT;
        p.KC = KC;
        p.hpitch = KC * 2 + 16;
        p.ksplit = (prefer_mfma && KC == d) ? ksplit : 1;
        p.nwaves = (prefer_mfma && KC == d) ? nwaves : NWx;
        p.extra_rows = (prefer_mfma && KC == d) ? extra_rows : 0;
        if (xany) p.extra_rows = Rx - vt::kMfmaTileRows;
        const int tile_rows = 16 * (p.nwaves / p.ksplit) + p.extra_rows;
        p.nlists = fixed.nwaves != 0 ? fixed.nlists : (k + tile_rows - 1) / tile_rows;
        p.L = m < tile_rows ? m : tile_rows;
        p.nblocks = p.nlists;
        p.lds = NT >= 8 ? stage : stage + ((n <= 8 ? 8 : 16 * (size_t)NT) + (xrows ? 16 : 0)) * p.hpitch;
        if (xrows) {
            p.xoff = (int)((p.lds + 15) & ~(size_t)15);
            p.lds = (size_t)p.xoff + xbytes;
        }
        // logit tile of the epilogue + 4 x 16 candidate keys per wave behind it
        // (+ the four range sums of 16 rows per hidden row that a pass after the march leaves)
        size_t tile = (((size_t)p.ksplit * n * (vt::kMfmaTileRows + (xany ? 17 : 1)) * sizeof(float) + 15) & ~(size_t)15) +
                      (size_t)vt::kStepWaves * 4 * 16 * sizeof(unsigned long long) +
                      (xpass ? (size_t)4 * n * 16 * sizeof(float) : 0);
        if (xrows && tile > (size_t)p.xoff) return p;      // (the extra rows' logits are read from behind the chunk into the tile)
        if (n <= vt::kStepWaves) {      // a wave per row: a candidate key per tile row and wave, not below 8 KiB
            const int tp = (p.extra_rows != 0 ? vt::kMfmaTileRows + 16 : p.nwaves == vt::kStepWaves ? vt::kMfmaTileRows : tile_rows) + 1;
            const size_t zt = ((size_t)p.ksplit * n * tp * sizeof(float) + 15) & ~(size_t)15;
            tile = (zt > 8192 ? zt : 8192) +
                   (size_t)p.nwaves * ((p.nwaves == vt::kStepWaves && p.extra_rows == 0) ? 2 : 3) * 64 * sizeof(unsigned long long) +
                   (p.extra_rows != 0 ? (size_t)8 * n * 16 * sizeof(float) : 0);      // + the shared group's partials
        }
        if (tile > p.lds) p.lds = tile;
        if (p.lds > (size_t)vt::kMaxDynamicLds) return p;
        const int group = p.nlists < vt::kStepMaxBlocks ? p.nlists : vt::kStepMaxBlocks;
        p.fin_stage_keys = (group + 1) * p.L;
        const int fc = (int)(vt::kFinalizeLdsBytes / ((size_t)p.fin_stage_keys * sizeof(unsigned long long)));
        // The per-tile candidate lists cost n * L selection rounds per tile and grow to megabytes; beyond a point
        // (measured: 12 or more tokens per row, or n * L from about 1280; always when the lists no longer fit the
        // merge's LDS staging) the kernel stores its logits instead and a workgroup per hidden row finishes the step.
        // With more than 8 hidden rows the tile epilogue selects by threshold only up to 8 tokens per row (four rows per
        // wave, 16 candidate slots each) and takes L rounds beyond: there the per-row tail wins from 9 tokens on
        // (measured, k = 32768, d = 4096: n = 64, m = 9: 58.4 against 60.1 us, m = 11: 58.5 / 61.8; n = 32, m = 10:
        // 53.8 / 55.1).
        const int max_list = n > vt::kGemvMaxN ? vt::kRowSelectMinLManyRows : vt::kRowSelectMinL;
        p.row_select = p.L > max_list || n * p.L >= vt::kRowSelectMinWork || fc < 1;
        // one hidden row per workgroup: n <= 256 rows spread over as many CUs, and a merging wave has its
        // SIMD to itself (the selection rounds are bound by instruction issue)
        p.fin_conc = 1;
        p.fin_lds = (size_t)p.fin_conc * p.fin_stage_keys * sizeof(unsigned long long);
        // (Merging in the main kernel's last workgroup to arrive was measured for n <= 8: 41.1 against 39.9 us --
        // eight merge workgroups on eight CUs beat eight waves on one; and for n <= 3 once more: 39.6 against 35.3.)
    } else {
        // many tokens per row: the selection rounds of the fused tail grow with L in every workgroup and the merge
        // stages B * L keys per row; the per-row tail on stored logits takes over (measured crossover)
        p.row_select = p.L > vt::kGemvRowSelectBase - n / 2;
    }

    size_t off = kTicketBytes;
    p.off_lse = off;
    off = round_up(off + (size_t)n * sizeof(float), 256);
    p.off_pms = off;
    off = round_up(off + (size_t)p.nblocks * n * sizeof(unsigned long long), 256);
    p.off_pkeys = off;
    off = round_up(off + (size_t)n * p.nblocks * p.L * sizeof(unsigned long long), 256);
    p.off_hpack = off;
    if (p.mfma && p.NT >= 8) off = round_up(off + (size_t)d * p.NT * 32, 256);
    p.off_zbuf = off;
    if (p.row_select) off = round_up(off + (size_t)n * k * sizeof(float), 256);
    p.bytes = off;
    p.ok = true;
    return p;
}

// Hidden rows handled per launch group.  A step whose n no single plan covers (more than 256 rows; more
// than 8 rows in fp32 or with d not a multiple of 128; very long fp32 rows) runs as consecutive groups
// of `chunk` rows, each streaming W_trim again -- slower, but every shape has an answer.
// Tree level fused behind the step (n <= 8 path only): null members = none.
struct TreeFuse {
    const float *cum = nullptr;
    int K = 0;
    int32_t *parent = nullptr;
    int32_t *token = nullptr;
    float *score = nullptr;
    // rows picked out of a larger batch (small-n kernel without the per-row tail only): hidden row i of the
    // group is row (row_pack >> 8 i) & 255 of h and of the outputs
    unsigned long long row_pack = 0;
    int indexed = 0;
};
int run_step_group(const void *h, int n, const void *W_trim, int w_type, int k, int d, const int32_t *map, int m,
                   int32_t *out_ids, float *out_logp, float *out_lse, float *out_logp_full, void *ws,
                   hipStream_t st, const TreeFuse &tf);

int pick_chunk(int n, int k, int d, int m, int dtype);

// several heads' tiles in one launch (defined with the launch code below)
constexpr int kNotFused = -1;
StepPlan plan_heads_fused(int n, int d, const int32_t *k, const int *used, int nused, int m, int w_type);
int run_step_heads_fused(const void *h, int n, int d, const void *const *W_trim, int w_type, const int32_t *k,
                         const int32_t *const *map, int n_heads, const int32_t *head_of_row, const vt::RowList *rows, int m,
                         int32_t *out_ids, float *out_logp, float *out_lse, void *ws, size_t ws_step_bytes, hipStream_t st);

// All n rows of a validated step: consecutive launch groups of `chunk` rows on one workspace.
int run_step_rows(const void *h, int n, const void *W_trim, int w_type, int k, int d, const int32_t *map, int m,
                  int32_t *out_ids, float *out_logp, float *out_lse, float *out_logp_full, void *ws, hipStream_t st) {
    const int chunk = pick_chunk(n, k, d, m, w_type);
    if (chunk == 0) return VT_ERR_SHAPE;
    const size_t row_bytes = (size_t)d * elem_size(w_type);
    for (int i0 = 0; i0 < n; i0 += chunk) {
        const int nc = n - i0 < chunk ? n - i0 : chunk;
        const int rc = run_step_group(static_cast<const char *>(h) + (size_t)i0 * row_bytes, nc, W_trim, w_type, k, d, map,
                                      m, out_ids + (size_t)i0 * m, out_logp + (size_t)i0 * m,
                                      out_lse ? out_lse + i0 : nullptr,
                                      out_logp_full ? out_logp_full + (size_t)i0 * k : nullptr, ws, st, TreeFuse{});
        if (rc != VT_OK) return rc;
    }
    return VT_OK;
}

// Workspace a step of up to n rows on a head of k rows may need, whatever the element type
size_t step_ws_bytes(int n, int k, int d, int m) {
    size_t b = 0;
    for (int dtype : {VT_BF16, VT_F32}) {
        const int c = pick_chunk(n, k, d, m, dtype);
        if (c == 0) continue;
        for (bool force_gemv : {false, true}) {      // either kernel may serve a group of up to 8 rows
            const StepPlan p = plan_step(c, k, d, m, dtype, force_gemv);
            if (p.ok && p.bytes > b) b = p.bytes;
            if (n % c != 0) {
                const StepPlan r = plan_step(n % c, k, d, m, dtype, force_gemv);
                if (r.ok && r.bytes > b) b = r.bytes;
            }
        }
    }
    return b;
}

// Layout of a multi-head workspace: the step workspace first, then the staged hidden rows and the staged results
// of one head's rows.
struct MultiLayout {
    size_t off_h = 0, off_ids = 0, off_logp = 0, off_lse = 0, bytes = 0;
};
MultiLayout multi_layout(int n, int d, const int32_t *k, int n_heads, int m) {
    // consecutive steps repeat their shapes: the last answer is kept per host thread
    struct Key {
        int n = 0, d = 0, m = 0, n_heads = 0;
        int32_t k[VT_MAX_HEADS] = {};
        MultiLayout L;
    };
    static thread_local Key last;
    if (last.n == n && last.d == d && last.m == m && last.n_heads == n_heads) {
        bool same = true;
        for (int hd = 0; hd < n_heads; ++hd) same = same && last.k[hd] == k[hd];
        if (same) return last.L;
    }
    MultiLayout L;
    size_t step = 0;
    for (int hd = 0; hd < n_heads; ++hd) {
        // a head may receive any number of the n rows, and the plan (hence its workspace) changes with it
        for (int nn = 1; nn <= n; ++nn) {
            const size_t b = step_ws_bytes(nn, k[hd], d, m);
            if (b > step) step = b;
        }
    }
    // ... and several heads' tiles in one launch: at most one tile per CU, whatever their shape
    if (n <= vt::kGemvMaxN) {
        for (int nw = vt::kStepWaves; nw <= vt::kMfmaMaxWaves; ++nw) {
            for (int ks = 1; ks <= (nw == vt::kStepWaves ? 4 : 1); ks *= 2) {
                FixedTiles ft;
                ft.nwaves = nw;
                ft.ksplit = ks;
                ft.nlists = vt::kStepMaxBlocks;
                const StepPlan p = plan_step_impl(n, vt::kStepMaxBlocks * 16 * (nw / ks), d, m, VT_BF16, false, ft);
                if (p.ok && p.bytes > step) step = p.bytes;
            }
        }
    }
    size_t off = round_up(step, 256);
    L.off_h = off;
    off = round_up(off + (size_t)n * d * sizeof(float), 256);      // sized for the wider element type
    L.off_ids = off;
    off = round_up(off + (size_t)n * m * sizeof(int32_t), 256);
    L.off_logp = off;
    off = round_up(off + (size_t)n * m * sizeof(float), 256);
    L.off_lse = off;
    off = round_up(off + (size_t)n * sizeof(float), 256);
    L.bytes = off;
    last.n = n;
    last.d = d;
    last.m = m;
    last.n_heads = n_heads;
    for (int hd = 0; hd < n_heads; ++hd) last.k[hd] = k[hd];
    last.L = L;
    return L;
}

int pick_chunk(int n, int k, int d, int m, int dtype) {
    if (plan_step(n, k, d, m, dtype).ok) return n;
    for (int c : {256, 8, 4, 2, 1}) {
        if (c < n && plan_step(c, k, d, m, dtype).ok && (n % c == 0 || plan_step(n % c, k, d, m, dtype).ok)) return c;
    }
    return 0;
}

}  // namespace

extern "C" {

const char *vt_status_string(int status) {
    switch (status) {
        case VT_OK: return "VT_OK";
        case VT_ERR_NULL: return "VT_ERR_NULL: a required pointer is NULL";
        case VT_ERR_SHAPE: return "VT_ERR_SHAPE: a size is out of range";
        case VT_ERR_DTYPE: return "VT_ERR_DTYPE: unknown or unsupported element or index type";
        case VT_ERR_ALIGN: return "VT_ERR_ALIGN: pointer or row size not 16-byte aligned";
        case VT_ERR_WORKSPACE: return "VT_ERR_WORKSPACE: workspace missing, misaligned or too small";
        case VT_ERR_DEVICE: return "VT_ERR_DEVICE: a HIP call failed";
        default: return "unknown vt_status";
    }
}

const char *vt_last_device_error(void) { return hipGetErrorString(g_last_hip_error); }

// ------------------------------------------------------------------ Algorithm 1
size_t vt_count_tokens_ws_bytes(int32_t V, int64_t n_ids) {
    if (V <= 0 || n_ids < 0) return 0;
    return round_up((size_t)vt::hist_num_chunks(n_ids, V) * (size_t)((V + 1) & ~1) * sizeof(unsigned short), 256);
}

int vt_count_tokens(const void *ids, int id_type, int64_t n_ids, int32_t V, int64_t *counts,
                    uint64_t *n_invalid, void *ws, size_t ws_bytes, void *stream) {
    if (id_type != VT_I32 && id_type != VT_I64) return VT_ERR_DTYPE;
    if (V <= 0 || n_ids < 0 || n_ids > ((int64_t)1 << 37)) return VT_ERR_SHAPE;
    if (counts == nullptr || (ids == nullptr && n_ids > 0)) return VT_ERR_NULL;
    if (n_ids == 0) return VT_OK;
    const size_t idb = id_type == VT_I64 ? 8 : 4;
    if (!aligned(ids, idb) || !aligned(counts, 8) || (n_invalid && !aligned(n_invalid, 8))) return VT_ERR_ALIGN;
    if (ws == nullptr || !aligned(ws, 256) || ws_bytes < vt_count_tokens_ws_bytes(V, n_ids)) return VT_ERR_WORKSPACE;
    (void)hipGetLastError();
    return device_status(vt::launch_count_tokens(ids, id_type == VT_I64, n_ids, V,
                                                 reinterpret_cast<long long *>(counts),
                                                 reinterpret_cast<unsigned long long *>(n_invalid),
                                                 static_cast<unsigned *>(ws), static_cast<hipStream_t>(stream)));
}

// ------------------------------------------------------------------ Eq. 1
size_t vt_build_trimmed_head_ws_bytes(int32_t V, int32_t d, int32_t k) {
    (void)d;
    (void)k;
    // the larger of: selection histograms (id order), buffers of a sort of all V (count, id) pairs (rank order)
    const size_t a = vt::select_scratch_bytes(V > 0 ? V : 1), b = vt::rank_sort_scratch_bytes(V > 0 ? V : 1);
    return 256 + round_up(a > b ? a : b, 256);
}

int vt_build_trimmed_head(const int64_t *counts, int32_t V, const void *W, int w_type, int32_t d, int32_t k,
                          int32_t *map, void *W_trim, void *ws, size_t ws_bytes, void *stream) {
    if (w_type != VT_F32 && w_type != VT_BF16) return VT_ERR_DTYPE;
    if (V <= 0 || d <= 0 || k < 1 || k > V) return VT_ERR_SHAPE;
    if (counts == nullptr || map == nullptr) return VT_ERR_NULL;
    if ((W == nullptr) != (W_trim == nullptr)) return VT_ERR_NULL;
    const size_t row_bytes = (size_t)d * elem_size(w_type);
    if (!aligned(counts, 8) || !aligned(map, 4)) return VT_ERR_ALIGN;
    if (W != nullptr && ((row_bytes & 15) != 0 || !aligned(W, 16) || !aligned(W_trim, 16))) return VT_ERR_ALIGN;
    if (ws == nullptr || !aligned(ws, 256) || ws_bytes < vt_build_trimmed_head_ws_bytes(V, d, k))
        return VT_ERR_WORKSPACE;
    (void)hipGetLastError();
    hipStream_t st = static_cast<hipStream_t>(stream);
    vt::launch_select_topk(reinterpret_cast<const long long *>(counts), V, k, static_cast<char *>(ws) + 256, map, st);
    if (W != nullptr) vt::launch_gather_rows(W, row_bytes, map, k, W_trim, st);
    return launch_status();
}

int vt_build_trimmed_head_by_rank(const int64_t *counts, int32_t V, const void *W, int w_type, int32_t d, int32_t k,
                                  int32_t *map, void *W_trim, void *ws, size_t ws_bytes, void *stream) {
    if (w_type != VT_F32 && w_type != VT_BF16) return VT_ERR_DTYPE;
    if (V <= 0 || d <= 0 || k < 1 || k > V) return VT_ERR_SHAPE;
    if (counts == nullptr || map == nullptr) return VT_ERR_NULL;
    if ((W == nullptr) != (W_trim == nullptr)) return VT_ERR_NULL;
    const size_t row_bytes = (size_t)d * elem_size(w_type);
    if (!aligned(counts, 8) || !aligned(map, 4)) return VT_ERR_ALIGN;
    if (W != nullptr && ((row_bytes & 15) != 0 || !aligned(W, 16) || !aligned(W_trim, 16))) return VT_ERR_ALIGN;
    if (ws == nullptr || !aligned(ws, 256) || ws_bytes < vt_build_trimmed_head_ws_bytes(V, d, k))
        return VT_ERR_WORKSPACE;
    (void)hipGetLastError();
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the k best ids in rank order are the first k of the full rank order
    vt::launch_rank_sort(reinterpret_cast<const long long *>(counts), V, static_cast<char *>(ws) + 256, map, k,
                         nullptr, st);
    if (W != nullptr) vt::launch_gather_rows(W, row_bytes, map, k, W_trim, st);
    return launch_status();
}

size_t vt_choose_k_ws_bytes(int32_t V) {
    if (V < 1) return 256;
    return round_up((size_t)V * sizeof(int32_t), 256) + round_up((size_t)V * sizeof(int64_t), 256) +
           vt::choose_k_scratch_bytes(V) + vt::rank_sort_scratch_bytes(V);
}

int vt_choose_k(const int64_t *counts, int32_t V, int mode, double p, int64_t min_count, int64_t *out, void *ws,
                size_t ws_bytes, void *stream) {
    if (mode != VT_K_TOP_P && mode != VT_K_MIN_COUNT) return VT_ERR_DTYPE;
    if (V <= 0) return VT_ERR_SHAPE;
    if (mode == VT_K_TOP_P && !(p >= 0.0 && p <= 1.0)) return VT_ERR_SHAPE;
    if (counts == nullptr || out == nullptr) return VT_ERR_NULL;
    if (!aligned(counts, 8) || !aligned(out, 8)) return VT_ERR_ALIGN;
    if (ws == nullptr || !aligned(ws, 256) || ws_bytes < vt_choose_k_ws_bytes(V)) return VT_ERR_WORKSPACE;
    (void)hipGetLastError();
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *wsb = static_cast<char *>(ws);
    int *ids = reinterpret_cast<int *>(wsb);
    long long *sorted = reinterpret_cast<long long *>(wsb + round_up((size_t)V * sizeof(int32_t), 256));
    char *bsum = wsb + round_up((size_t)V * sizeof(int32_t), 256) + round_up((size_t)V * sizeof(int64_t), 256);
    void *scratch = bsum + vt::choose_k_scratch_bytes(V);
    const long long *c = reinterpret_cast<const long long *>(counts);
    vt::launch_rank_sort(c, V, scratch, ids, V, sorted, st);
    vt::launch_choose_k(sorted, V, mode, p, (long long)min_count, bsum, reinterpret_cast<long long *>(out), st);
    return launch_status();
}

// ------------------------------------------------------------------ Algorithm 2, drafting lines
size_t vt_draft_head_step_ws_bytes(int32_t n, int32_t k, int32_t d, int32_t m) {
    return step_ws_bytes(n, k, d, m);      // sized for either element type
}

int vt_draft_head_step_plan(int32_t n, int32_t k, int32_t d, int32_t m, int w_type, char *text, size_t text_bytes) {
    if (w_type != VT_F32 && w_type != VT_BF16) return VT_ERR_DTYPE;
    if (n <= 0 || k <= 0 || d <= 0 || m < 1 || m > k || m > VT_MAX_TOP_M || k > vt::kStepMaxK) return VT_ERR_SHAPE;
    if (text == nullptr || text_bytes == 0) return VT_ERR_NULL;
    const int chunk = pick_chunk(n, k, d, m, w_type);
    if (chunk == 0) return VT_ERR_SHAPE;
    const StepPlan p = plan_step(chunk, k, d, m, w_type);
    if (!p.ok) return VT_ERR_SHAPE;
    char head[160];
    if (p.gemv) {
        std::snprintf(head, sizeof head, "head_gemv_kernel<%s,%d,%d> workgroups=%d rows_per_workgroup=%d column_segments=%d",
                      w_type == VT_BF16 ? "bf16" : "f32", p.NP, p.CS, p.nblocks, p.rpb, p.S);
    } else if (p.NT >= 8) {
        std::snprintf(head, sizeof head, "pack_h_kernel + head_mfma_wide_kernel<%d> workgroups=%d tile_rows=%d", p.NT / 8,
                      p.nlists, vt::kMfmaTileRows);
    } else {
        std::snprintf(head, sizeof head, "head_mfma_kernel<%d,%d> workgroups=%d tile_rows=%d waves=%d column_split=%d", p.NT,
                      p.nwaves == vt::kStepWaves ? vt::kStepWaves : p.NT > 1 ? vt::kMfmaFewWaves : vt::kMfmaMaxWaves, p.nlists,
                      16 * (p.nwaves / p.ksplit) + p.extra_rows, p.nwaves, p.ksplit);
    }
    const char *tail = p.row_select ? " + row_select_kernel" : " + step_finalize_kernel";
    char groups[48] = "";
    if (chunk < n) std::snprintf(groups, sizeof groups, " x %d row groups", (n + chunk - 1) / chunk);
    std::snprintf(text, text_bytes, "%s%s%s", head, tail, groups);
    return VT_OK;
}

int vt_draft_head_step_multi_plan(int32_t n, int32_t d, const int32_t *k, int32_t n_heads, const int32_t *head_of_row,
                                  int32_t m, int w_type, char *text, size_t text_bytes) {
    if (w_type != VT_F32 && w_type != VT_BF16) return VT_ERR_DTYPE;
    if (n < 1 || n > VT_MULTI_MAX_ROWS || d < 1 || n_heads < 1 || n_heads > VT_MAX_HEADS) return VT_ERR_SHAPE;
    if (k == nullptr || head_of_row == nullptr || text == nullptr || text_bytes == 0) return VT_ERR_NULL;
    int rows_of[VT_MAX_HEADS] = {};
    for (int i = 0; i < n; ++i) {
        if (head_of_row[i] < 0 || head_of_row[i] >= n_heads) return VT_ERR_SHAPE;
        ++rows_of[head_of_row[i]];
    }
    int used[VT_MAX_HEADS], nused = 0;
    for (int hd = 0; hd < n_heads; ++hd) {
        if (k[hd] < 1 || k[hd] > vt::kStepMaxK) return VT_ERR_SHAPE;
        if (rows_of[hd] == 0) continue;
        if (m < 1 || m > k[hd] || m > VT_MAX_TOP_M) return VT_ERR_SHAPE;
        used[nused++] = hd;
    }
    const StepPlan p = plan_heads_fused(n, d, k, used, nused, m, w_type);
    if (p.ok) {
        std::snprintf(text, text_bytes,
                      "head_mfma_kernel<1,%d> heads=%d workgroups=%d tile_rows=%d waves=%d column_split=%d + step_finalize_kernel",
                      p.nwaves == vt::kStepWaves ? vt::kStepWaves : vt::kMfmaMaxWaves, nused, p.nlists,
                      16 * (p.nwaves / p.ksplit), p.nwaves, p.ksplit);
    } else {
        std::snprintf(text, text_bytes, "head by head (%d)", nused);
    }
    return VT_OK;
}

int vt_draft_head_step_ws_init(void *ws, size_t ws_bytes, void *stream) {
    if (ws == nullptr || !aligned(ws, 256) || ws_bytes < kTicketBytes) return VT_ERR_WORKSPACE;
    (void)hipGetLastError();
    vt::launch_ws_clear(static_cast<unsigned *>(ws), (int)(kTicketBytes / sizeof(unsigned)),
                        static_cast<hipStream_t>(stream));
    return launch_status();
}

int vt_draft_head_step(const void *h, int h_type, int32_t n, const void *W_trim, int w_type, int32_t k, int32_t d,
                       const int32_t *map, int32_t m, int32_t *out_ids, float *out_logp, float *out_lse,
                       float *out_logp_full, void *ws, size_t ws_bytes, void *stream) {
    if ((h_type != VT_F32 && h_type != VT_BF16) || (w_type != VT_F32 && w_type != VT_BF16)) return VT_ERR_DTYPE;
    if (h_type != w_type) return VT_ERR_DTYPE;
    if (n <= 0 || k <= 0 || d <= 0 || k > vt::kStepMaxK) return VT_ERR_SHAPE;
    if (m < 1 || m > k || m > VT_MAX_TOP_M) return VT_ERR_SHAPE;
    if (h == nullptr || W_trim == nullptr || map == nullptr || out_ids == nullptr || out_logp == nullptr)
        return VT_ERR_NULL;
    const size_t row_bytes = (size_t)d * elem_size(w_type);
    if ((row_bytes & 15) != 0 || !aligned(h, 16) || !aligned(W_trim, 16) || !aligned(map, 4) ||
        !aligned(out_ids, 4) || !aligned(out_logp, 4) || (out_lse && !aligned(out_lse, 4)) ||
        (out_logp_full && !aligned(out_logp_full, 4)))
        return VT_ERR_ALIGN;
    if (pick_chunk(n, k, d, m, w_type) == 0) return VT_ERR_SHAPE;
    if (ws == nullptr || !aligned(ws, 256) || ws_bytes < vt_draft_head_step_ws_bytes(n, k, d, m))
        return VT_ERR_WORKSPACE;
    (void)hipGetLastError();
    const int rc = run_step_rows(h, n, W_trim, w_type, k, d, map, m, out_ids, out_logp, out_lse, out_logp_full, ws,
                                 static_cast<hipStream_t>(stream));
    if (rc != VT_OK) return rc;
    return launch_status();
}

int vt_draft_head_step_static(const void *h, int h_type, int32_t n, const void *W_trim, int w_type, int32_t k,
                              int32_t d, const int32_t *map, int32_t m, int32_t *out_ids, float *out_logp,
                              float *out_lse, float *out_logp_full, void *stream) {
    // the size check comes first and touches no device: a shape is either out of range altogether (0) or needs
    // more than the library's own array holds
    if (n <= 0 || k <= 0 || d <= 0 || m < 1) return VT_ERR_SHAPE;
    const size_t need = vt_draft_head_step_ws_bytes(n, k, d, m);
    if (need == 0) return VT_ERR_SHAPE;
    if (need > (size_t)VT_STATIC_WS_BYTES) return VT_ERR_WORKSPACE;
    void *ws = nullptr;
    const int rc = static_scratch_of_current_device(&ws);
    if (rc != VT_OK) return rc;
    // Nothing has to be cleared here: a step rewrites everything it reads in the array before it reads it (the
    // one counted word, the ticket of a fused tree level, is zeroed by the kernel that runs before its user).
    return vt_draft_head_step(h, h_type, n, W_trim, w_type, k, d, map, m, out_ids, out_logp, out_lse, out_logp_full,
                              ws, (size_t)VT_STATIC_WS_BYTES, stream);
}

// ------------------------------------------------------------------ several heads in one step
size_t vt_draft_head_step_multi_ws_bytes(int32_t n, int32_t d, const int32_t *k, int32_t n_heads, int32_t m) {
    if (n < 1 || n > VT_MULTI_MAX_ROWS || d < 1 || k == nullptr || n_heads < 1 || n_heads > VT_MAX_HEADS || m < 1)
        return 0;
    for (int hd = 0; hd < n_heads; ++hd) {
        if (k[hd] < 1 || k[hd] > vt::kStepMaxK) return 0;
    }
    return multi_layout(n, d, k, n_heads, m).bytes;
}

int vt_draft_head_step_multi(const void *h, int h_type, int32_t n, int32_t d, const void *const *W_trim, int w_type,
                             const int32_t *k, const int32_t *const *map, int32_t n_heads,
                             const int32_t *head_of_row, int32_t m, int32_t *out_ids, float *out_logp,
                             float *out_lse, void *ws, size_t ws_bytes, void *stream) {
    if ((h_type != VT_F32 && h_type != VT_BF16) || (w_type != VT_F32 && w_type != VT_BF16)) return VT_ERR_DTYPE;
    if (h_type != w_type) return VT_ERR_DTYPE;
    if (n < 1 || n > VT_MULTI_MAX_ROWS || d < 1 || n_heads < 1 || n_heads > VT_MAX_HEADS) return VT_ERR_SHAPE;
    if (h == nullptr || W_trim == nullptr || k == nullptr || map == nullptr || head_of_row == nullptr ||
        out_ids == nullptr || out_logp == nullptr)
        return VT_ERR_NULL;
    const size_t row_bytes = (size_t)d * elem_size(w_type);
    if ((row_bytes & 15) != 0 || !aligned(h, 16) || !aligned(out_ids, 4) || !aligned(out_logp, 4) ||
        (out_lse && !aligned(out_lse, 4)))
        return VT_ERR_ALIGN;
    // rows of every head, in ascending row order
    vt::RowList rows[VT_MAX_HEADS];
    for (int hd = 0; hd < n_heads; ++hd) rows[hd].n = 0;
    for (int i = 0; i < n; ++i) {
        const int hd = head_of_row[i];
        if (hd < 0 || hd >= n_heads) return VT_ERR_SHAPE;
        rows[hd].idx[rows[hd].n++] = (short)i;
    }
    for (int hd = 0; hd < n_heads; ++hd) {
        if (k[hd] < 1 || k[hd] > vt::kStepMaxK) return VT_ERR_SHAPE;
        if (rows[hd].n == 0) continue;           // an unused head needs no valid pointers
        if (m < 1 || m > k[hd] || m > VT_MAX_TOP_M) return VT_ERR_SHAPE;
        if (W_trim[hd] == nullptr || map[hd] == nullptr) return VT_ERR_NULL;
        if (!aligned(W_trim[hd], 16) || !aligned(map[hd], 4)) return VT_ERR_ALIGN;
        if (pick_chunk(rows[hd].n, k[hd], d, m, w_type) == 0) return VT_ERR_SHAPE;
    }
    const MultiLayout L = multi_layout(n, d, k, n_heads, m);
    if (ws == nullptr || !aligned(ws, 256) || ws_bytes < L.bytes) return VT_ERR_WORKSPACE;
    (void)hipGetLastError();
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *wsb = static_cast<char *>(ws);
    {
        const int rc = run_step_heads_fused(h, n, d, W_trim, w_type, k, map, n_heads, head_of_row, rows, m, out_ids, out_logp,
                                            out_lse, ws, L.off_h, st);
        if (rc != kNotFused) return rc == VT_OK ? launch_status() : rc;
    }
    for (int hd = 0; hd < n_heads; ++hd) {
        const vt::RowList &R = rows[hd];
        if (R.n == 0) continue;
        const int first = R.idx[0];
        const bool consecutive = R.idx[R.n - 1] - first == R.n - 1;
        if (consecutive) {
            // the head's rows lie next to each other in h: the step reads and writes them in place
            const int rc = run_step_rows(static_cast<const char *>(h) + (size_t)first * row_bytes, R.n, W_trim[hd], w_type,
                                         k[hd], d, map[hd], m, out_ids + (size_t)first * m, out_logp + (size_t)first * m,
                                         out_lse ? out_lse + first : nullptr, nullptr, ws, st);
            if (rc != VT_OK) return rc;
            continue;
        }
        const StepPlan plan = plan_step(R.n, k[hd], d, m, w_type);
        if (R.n <= vt::kGemvMaxN && plan.ok && !plan.row_select) {
            // few rows: the kernel picks its hidden rows out of h and writes their output rows itself
            TreeFuse pick;
            pick.indexed = 1;
            for (int i = 0; i < R.n; ++i) pick.row_pack |= (unsigned long long)(R.idx[i] & 0xFF) << (8 * i);
            const int rc = run_step_group(h, R.n, W_trim[hd], w_type, k[hd], d, map[hd], m, out_ids, out_logp, out_lse,
                                          nullptr, ws, st, pick);
            if (rc != VT_OK) return rc;
            continue;
        }
        int32_t *ids_s = reinterpret_cast<int32_t *>(wsb + L.off_ids);
        float *logp_s = reinterpret_cast<float *>(wsb + L.off_logp);
        float *lse_s = reinterpret_cast<float *>(wsb + L.off_lse);
        vt::launch_gather_h_rows(h, wsb + L.off_h, row_bytes, R, st);
        const int rc = run_step_rows(wsb + L.off_h, R.n, W_trim[hd], w_type, k[hd], d, map[hd], m, ids_s, logp_s, lse_s,
                                     nullptr, ws, st);
        if (rc != VT_OK) return rc;
        vt::launch_scatter_rows(ids_s, logp_s, lse_s, m, out_ids, out_logp, out_lse, R, st);
    }
    return launch_status();
}

// ------------------------------------------------------------------ several heads built from one W
int vt_build_trimmed_heads(const int64_t *counts, int32_t V, int32_t n_heads, const void *W, int w_type, int32_t d,
                           const int32_t *k, int32_t *const *map, void *const *W_trim, void *ws, size_t ws_bytes,
                           void *stream) {
    if (n_heads < 1 || n_heads > VT_MAX_HEADS) return VT_ERR_SHAPE;
    if (counts == nullptr || k == nullptr || map == nullptr) return VT_ERR_NULL;
    if ((W == nullptr) != (W_trim == nullptr)) return VT_ERR_NULL;
    if (V <= 0) return VT_ERR_SHAPE;
    // every head is checked before the first one is built
    for (int hd = 0; hd < n_heads; ++hd) {
        if (k[hd] < 1 || k[hd] > V) return VT_ERR_SHAPE;
        if (map[hd] == nullptr || (W != nullptr && W_trim[hd] == nullptr)) return VT_ERR_NULL;
        if (ws_bytes < vt_build_trimmed_head_ws_bytes(V, d, k[hd])) return VT_ERR_WORKSPACE;
    }
    // the checks of the single-head build, for every head
    if (w_type != VT_F32 && w_type != VT_BF16) return VT_ERR_DTYPE;
    if (d <= 0) return VT_ERR_SHAPE;
    const size_t row_bytes = (size_t)d * elem_size(w_type);
    if (!aligned(counts, 8)) return VT_ERR_ALIGN;
    if (W != nullptr && ((row_bytes & 15) != 0 || !aligned(W, 16))) return VT_ERR_ALIGN;
    for (int hd = 0; hd < n_heads; ++hd) {
        if (!aligned(map[hd], 4) || (W != nullptr && !aligned(W_trim[hd], 16))) return VT_ERR_ALIGN;
    }
    if (ws == nullptr || !aligned(ws, 256)) return VT_ERR_WORKSPACE;
    static_assert(VT_MAX_HEADS == vt::kSelectMaxHeads, "heads per batched launch");
    (void)hipGetLastError();
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (256 + (size_t)n_heads * vt::select_scratch_stride(V) <= ws_bytes) {
        // all heads together: the selection's eleven launches and the row copy once, with the head as grid.y
        // (the selection is bound by its launches: 60 us for one head or sixteen)
        vt::launch_select_topk_heads(reinterpret_cast<const long long *>(counts), V, n_heads, k,
                                     static_cast<char *>(ws) + 256, map, st);
        if (W != nullptr)
            vt::launch_gather_rows_heads(W, row_bytes, n_heads, k, const_cast<const int *const *>(map), W_trim, st);
        return launch_status();
    }
    for (int hd = 0; hd < n_heads; ++hd) {
        const int rc = vt_build_trimmed_head(counts + (size_t)hd * V, V, W, w_type, d, k[hd], map[hd],
                                             W != nullptr ? W_trim[hd] : nullptr, ws, ws_bytes, stream);
        if (rc != VT_OK) return rc;
    }
    return VT_OK;
}

int vt_draft_tree_level(const void *h, int h_type, int32_t n, const void *W_trim, int w_type, int32_t k, int32_t d,
                        const int32_t *map, int32_t m, const float *parent_cum, int32_t K, int32_t *out_parent,
                        int32_t *out_token, float *out_cum, int32_t *out_ids, float *out_logp, void *ws,
                        size_t ws_bytes, void *stream) {
    if ((h_type != VT_F32 && h_type != VT_BF16) || (w_type != VT_F32 && w_type != VT_BF16)) return VT_ERR_DTYPE;
    if (h_type != w_type) return VT_ERR_DTYPE;
    if (n <= 0 || k <= 0 || d <= 0 || k > vt::kStepMaxK) return VT_ERR_SHAPE;
    if (m < 1 || m > k || m > VT_MAX_TOP_M) return VT_ERR_SHAPE;
    if ((int64_t)n * m > VT_TREE_MAX_CANDIDATES || K < 1 || (int64_t)K > (int64_t)n * m) return VT_ERR_SHAPE;
    if (h == nullptr || W_trim == nullptr || map == nullptr || out_ids == nullptr || out_logp == nullptr ||
        parent_cum == nullptr || out_parent == nullptr || out_token == nullptr || out_cum == nullptr)
        return VT_ERR_NULL;
    const size_t row_bytes = (size_t)d * elem_size(w_type);
    if ((row_bytes & 15) != 0 || !aligned(h, 16) || !aligned(W_trim, 16) || !aligned(map, 4) ||
        !aligned(out_ids, 4) || !aligned(out_logp, 4) || !aligned(parent_cum, 4) || !aligned(out_parent, 4) ||
        !aligned(out_token, 4) || !aligned(out_cum, 4))
        return VT_ERR_ALIGN;
    const int chunk = pick_chunk(n, k, d, m, w_type);
    if (chunk == 0) return VT_ERR_SHAPE;
    if (ws == nullptr || !aligned(ws, 256) || ws_bytes < vt_draft_head_step_ws_bytes(n, k, d, m))
        return VT_ERR_WORKSPACE;
    (void)hipGetLastError();
    hipStream_t st = static_cast<hipStream_t>(stream);
    // one launch when the small-n kernel covers the whole step: its last workgroup also ranks the candidates
    // (the same kernel as vt_draft_head_step would use for this shape, so both calls return the same bits)
    // ... or, on the matrix-core path, when its merge kernel (one workgroup per hidden row) covers all rows: the
    // workgroup that finishes last ranks the candidates
    const StepPlan small = plan_step(n, k, d, m, w_type);
    const bool fuse_gemv = small.ok && small.gemv && n * m <= vt::kStepWaves * 64;
    const bool fuse_mfma = small.ok && small.mfma && !small.row_select && chunk >= n && n * m <= vt::kFinalizeTreeMaxN;
    if (fuse_gemv || fuse_mfma) {
        TreeFuse tf;
        tf.cum = parent_cum;
        tf.K = K;
        tf.parent = out_parent;
        tf.token = out_token;
        tf.score = out_cum;
        const int rc = run_step_group(h, n, W_trim, w_type, k, d, map, m, out_ids, out_logp, nullptr, nullptr, ws, st, tf);
        if (rc != VT_OK) return rc;
        return launch_status();
    }
    for (int i0 = 0; i0 < n; i0 += chunk) {
        const int nc = n - i0 < chunk ? n - i0 : chunk;
        const int rc = run_step_group(static_cast<const char *>(h) + (size_t)i0 * row_bytes, nc, W_trim, w_type, k, d, map,
                                      m, out_ids + (size_t)i0 * m, out_logp + (size_t)i0 * m, nullptr, nullptr, ws, st,
                                      TreeFuse{});
        if (rc != VT_OK) return rc;
    }
    vt::TreeArgs a;
    a.parent_cum = parent_cum;
    a.vals = out_logp;
    a.ids = out_ids;
    a.N = n * m;
    a.m = m;
    a.K = K;
    a.index_order = 0;
    a.out_a = out_parent;
    a.out_token = out_token;
    a.out_score = out_cum;
    return device_status(vt::launch_tree_select(a, st));
}

}  // extern "C"

namespace {

// One launch group of the draft step: n rows that a single plan covers.  Arguments are validated.
// Up to 8 hidden rows on two or more heads: one launch of the matrix-core kernel over all those heads' tiles -- every
// head streams once and the fixed costs of a step (launches, epilogue, merge) are paid once, not per head -- then
// the merge kernel.  All tiles have one height, the smallest for which every head, cut on its own, fits one tile
// per CU in all: 32, 64 or 128 rows with eight waves (4, 2, 1 waves per 16-row group), 144 .. 192 rows with 9 .. 12
// waves.  Returns kNotFused where that does not apply (the caller then runs the heads one after another).
// The plan of that launch (ok = false where it does not apply): used = the heads that have rows.
StepPlan plan_heads_fused(int n, int d, const int32_t *k, const int *used, int nused, int m, int w_type) {
    StepPlan p;
    if (n > vt::kGemvMaxN || w_type != VT_BF16 || nused < 2) return p;
    const int CUS = round_workgroups();
    static const int shapes[][2] = {{8, 4}, {8, 2}, {8, 1}, {9, 1}, {10, 1}, {11, 1}, {12, 1}};
    for (const auto &sh : shapes) {
        const int T = 16 * (sh[0] / sh[1]);
        int tiles = 0;
        for (int q = 0; q < nused; ++q) tiles += (k[used[q]] + T - 1) / T;
        if (tiles > CUS) continue;
        FixedTiles ft;
        ft.nwaves = sh[0];
        ft.ksplit = sh[1];
        ft.nlists = tiles;
        p = plan_step_impl(n, tiles * T, d, m, w_type, false, ft);
        if (p.ok) break;
    }
    if (p.ok && (!p.mfma || p.row_select || p.KC != d || p.NT != 1)) p.ok = false;
    return p;
}
int run_step_heads_fused(const void *h, int n, int d, const void *const *W_trim, int w_type, const int32_t *k,
                         const int32_t *const *map, int n_heads, const int32_t *head_of_row, const vt::RowList *rows, int m,
                         int32_t *out_ids, float *out_logp, float *out_lse, void *ws, size_t ws_step_bytes, hipStream_t st) {
    int used[VT_MAX_HEADS], nused = 0;
    for (int hd = 0; hd < n_heads; ++hd)
        if (rows[hd].n != 0) used[nused++] = hd;
    const StepPlan p = plan_heads_fused(n, d, k, used, nused, m, w_type);
    if (!p.ok || p.bytes > ws_step_bytes) return kNotFused;
    const int T = 16 * (p.nwaves / p.ksplit);
    vt::MultiHeadTable t{};
    t.n_heads = nused;
    t.tile_first[0] = 0;
    int slot_of_head[VT_MAX_HEADS];
    for (int q = 0; q < nused; ++q) {
        const int hd = used[q];
        slot_of_head[hd] = q;
        t.W[q] = W_trim[hd];
        t.map[q] = map[hd];
        t.k[q] = k[hd];
        t.tile_first[q + 1] = t.tile_first[q] + (k[hd] + T - 1) / T;
    }
    for (int i = 0; i < n; ++i) t.head_of_row |= (unsigned long long)slot_of_head[head_of_row[i]] << (8 * i);
    char *wsb = static_cast<char *>(ws);
    vt::MfmaArgs a{};
    a.h = h;
    a.n = n;
    a.d = d;
    a.m = m;
    a.L = p.L;
    a.nlists = p.nlists;
    a.KC = p.KC;
    a.hpitch = p.hpitch;
    a.pms = reinterpret_cast<unsigned long long *>(wsb + p.off_pms);
    a.pkeys = reinterpret_cast<unsigned long long *>(wsb + p.off_pkeys);
    a.ksplit = p.ksplit;
    a.nwaves = p.nwaves;
    hipError_t e = vt::launch_head_mfma_multi(a, t, p.lds, st);
    if (e != hipSuccess) return device_status(e);
    vt::FinalizeArgs f{};
    f.pms = a.pms;
    f.pkeys = a.pkeys;
    f.nlists = p.nlists;
    f.L = p.L;
    f.n = n;
    f.m = m;
    f.conc = p.fin_conc;
    f.stage_keys = p.fin_stage_keys;
    f.out_ids = out_ids;
    f.out_logp = out_logp;
    f.out_lse = out_lse;
    f.lse_buf = reinterpret_cast<float *>(wsb + p.off_lse);
    f.ticket = reinterpret_cast<unsigned *>(wsb);
    e = vt::launch_step_finalize(f, p.fin_lds, st);
    return e == hipSuccess ? VT_OK : device_status(e);
}

int run_step_group(const void *h, int n, const void *W_trim, int w_type, int k, int d, const int32_t *map, int m,
                   int32_t *out_ids, float *out_logp, float *out_lse, float *out_logp_full, void *ws,
                   hipStream_t st, const TreeFuse &tf) {
    const StepPlan p = plan_step(n, k, d, m, w_type);
    if (!p.ok) return VT_ERR_SHAPE;
    char *wsb = static_cast<char *>(ws);
    unsigned long long *pms = reinterpret_cast<unsigned long long *>(wsb + p.off_pms);
    unsigned long long *pkeys = reinterpret_cast<unsigned long long *>(wsb + p.off_pkeys);
    float *lse_buf = reinterpret_cast<float *>(wsb + p.off_lse);
    if (p.gemv) {
        vt::StepArgs a;
        a.h = h;
        a.W = W_trim;
        a.map = map;
        a.n = n;
        a.k = k;
        a.d = d;
        a.m = m;
        a.S = p.S;
        a.rpb = p.rpb;
        a.tpitch = p.tpitch;
        a.L = p.L;
        a.nblocks = p.nblocks;
        a.pms = pms;
        a.pkeys = pkeys;
        a.out_logp_full = out_logp_full;
        a.zbuf = nullptr;
        if (p.row_select) a.zbuf = out_logp_full != nullptr ? out_logp_full : reinterpret_cast<float *>(wsb + p.off_zbuf);
        if (tf.indexed && (p.row_select || out_logp_full != nullptr)) return VT_ERR_SHAPE;
        a.row_pack = tf.indexed ? tf.row_pack : 0x0706050403020100ull;
        // a tree level fused behind the merge kernel: rows in order, at most kFinalizeTreeMaxN candidates
        const bool tree_behind_merge = tf.cum != nullptr && !p.row_select;
        if (tree_behind_merge && (tf.indexed || n * m > vt::kFinalizeTreeMaxN)) return VT_ERR_SHAPE;
        a.ticket_clear = tree_behind_merge ? reinterpret_cast<unsigned *>(wsb) : nullptr;
        const size_t lds = p.lds;
        const bool bf16 = w_type == VT_BF16;
        hipError_t e = hipErrorInvalidValue;
        switch (p.NP) {
            case 1: e = vt::launch_head_gemv_np1(bf16, p.CS, a, lds, st); break;
            case 2: e = vt::launch_head_gemv_np2(bf16, p.CS, a, lds, st); break;
            case 4: e = vt::launch_head_gemv_np4(bf16, p.CS, a, lds, st); break;
            case 8: e = vt::launch_head_gemv_np8(bf16, p.CS, a, lds, st); break;
            default: break;
        }
        if (e != hipSuccess) return device_status(e);
        if (!p.row_select) {
            vt::FinalizeArgs f{};
            f.pms = pms;
            f.pkeys = pkeys;
            f.nlists = p.nblocks;
            f.L = p.L;
            f.n = n;
            f.m = m;
            f.conc = 1;
            f.stage_keys = (p.nblocks + 1) * p.L;
            f.out_ids = out_ids;
            f.out_logp = out_logp;
            f.out_lse = out_lse;
            f.lse_buf = lse_buf;
            f.row_pack = tf.row_pack;
            f.indexed = tf.indexed;
            f.tree_cum = tf.cum;
            f.tree_K = tf.K;
            f.tree_parent = tf.parent;
            f.tree_token = tf.token;
            f.tree_score = tf.score;
            f.ticket = reinterpret_cast<unsigned *>(wsb);
            e = vt::launch_step_finalize(f, (size_t)f.stage_keys * sizeof(unsigned long long), st);
            if (e != hipSuccess) return device_status(e);
        }
        if (p.row_select) {
            vt::launch_row_select(a.zbuf, map, n, k, m, out_ids, out_logp, out_lse, lse_buf, st);
            if (out_logp_full != nullptr) vt::launch_sub_lse(out_logp_full, lse_buf, n, k, st);
            if (tf.cum != nullptr) {       // the fused tree level needs the merge kernel: run the expansion kernel
                vt::TreeArgs t;
                t.parent_cum = tf.cum;
                t.vals = out_logp;
                t.ids = out_ids;
                t.N = n * m;
                t.m = m;
                t.K = tf.K;
                t.index_order = 0;
                t.out_a = tf.parent;
                t.out_token = tf.token;
                t.out_score = tf.score;
                return device_status(vt::launch_tree_select(t, st));
            }
            return VT_OK;
        }
    } else {
        // a fused tree level needs the merge kernel (no per-row tail) and at most kFinalizeTreeMaxN candidates; row
        // picking needs up to 8 rows and the merge kernel too
        if ((tf.cum != nullptr && (p.row_select || tf.indexed || n * m > vt::kFinalizeTreeMaxN)) ||
            (tf.indexed && (n > vt::kGemvMaxN || p.row_select || out_logp_full != nullptr)))
            return VT_ERR_SHAPE;
        vt::MfmaArgs a;
        a.h = h;
        a.W = W_trim;
        a.map = map;
        a.n = n;
        a.k = k;
        a.d = d;
        a.m = m;
        a.L = p.L;
        a.nlists = p.nlists;
        a.KC = p.KC;
        a.hpitch = p.hpitch;
        a.pms = pms;
        a.pkeys = pkeys;
        a.out_logp_full = out_logp_full;
        a.hpack = p.NT >= 8 ? static_cast<void *>(wsb + p.off_hpack) : nullptr;
        a.zbuf = nullptr;
        if (p.row_select) a.zbuf = out_logp_full != nullptr ? out_logp_full : reinterpret_cast<float *>(wsb + p.off_zbuf);
        a.row_pack = tf.row_pack;
        a.indexed = tf.indexed;
        a.ksplit = p.ksplit;
        a.nwaves = p.nwaves;
        a.extra_rows = p.extra_rows;
        a.xoff = p.xoff;
        a.ticket_clear = tf.cum != nullptr ? reinterpret_cast<unsigned *>(wsb) : nullptr;
        hipError_t e = vt::launch_head_mfma(p.NT, a, p.lds, st);
        if (e != hipSuccess) return device_status(e);
        if (p.row_select) {
            vt::launch_row_select(a.zbuf, map, n, k, m, out_ids, out_logp, out_lse, lse_buf, st);
            if (out_logp_full != nullptr) vt::launch_sub_lse(out_logp_full, lse_buf, n, k, st);
            return VT_OK;
        }
        vt::FinalizeArgs f{};
        f.row_pack = tf.row_pack;
        f.indexed = tf.indexed;
        f.pms = pms;
        f.pkeys = pkeys;
        f.nlists = p.nlists;
        f.L = p.L;
        f.n = n;
        f.m = m;
        f.conc = p.fin_conc;
        f.stage_keys = p.fin_stage_keys;
        f.out_ids = out_ids;
        f.out_logp = out_logp;
        f.out_lse = out_lse;
        f.lse_buf = lse_buf;
        f.tree_cum = tf.cum;
        f.tree_K = tf.K;
        f.tree_parent = tf.parent;
        f.tree_token = tf.token;
        f.tree_score = tf.score;
        f.ticket = reinterpret_cast<unsigned *>(wsb);
        if (tf.cum != nullptr && (n * m > vt::kFinalizeTreeMaxN || tf.indexed)) return VT_ERR_SHAPE;
        e = vt::launch_step_finalize(f, p.fin_lds, st);
        if (e != hipSuccess) return device_status(e);
    }
    if (out_logp_full != nullptr)
        vt::launch_sub_lse(out_logp_full, lse_buf, n, k, st);
    return VT_OK;
}

}  // namespace

extern "C" {

int vt_tree_expand(const float *parent_cum, const float *step_logp, const int32_t *step_ids, int32_t n, int32_t m,
                   int32_t K, int32_t *out_parent, int32_t *out_token, float *out_cum, void *stream) {
    if (!parent_cum || !step_logp || !step_ids || !out_parent || !out_token || !out_cum) return VT_ERR_NULL;
    if (n < 1 || m < 1 || (int64_t)n * m > VT_TREE_MAX_CANDIDATES || K < 1 || K > n * m) return VT_ERR_SHAPE;
    vt::TreeArgs a;
    a.parent_cum = parent_cum;
    a.vals = step_logp;
    a.ids = step_ids;
    a.N = n * m;
    a.m = m;
    a.K = K;
    a.index_order = 0;
    a.out_a = out_parent;
    a.out_token = out_token;
    a.out_score = out_cum;
    return device_status(vt::launch_tree_select(a, static_cast<hipStream_t>(stream)));
}

int vt_tree_rerank(const float *cum, int32_t N, int32_t T, int32_t *out_idx, void *stream) {
    if (!cum || !out_idx) return VT_ERR_NULL;
    if (N < 1 || N > VT_TREE_MAX_CANDIDATES || T < 1 || T > N || T > VT_TREE_MAX_KEEP) return VT_ERR_SHAPE;
    static_assert(VT_TREE_MAX_CANDIDATES == vt::kTreeMaxN && VT_TREE_MAX_KEEP == vt::kTreeMaxKeepSorted, "limits");
    vt::TreeArgs a;
    a.parent_cum = nullptr;
    a.vals = cum;
    a.ids = nullptr;
    a.N = N;
    a.m = 1;
    a.K = T;
    a.index_order = 1;
    a.out_a = out_idx;
    a.out_token = nullptr;
    a.out_score = nullptr;
    return device_status(vt::launch_tree_select(a, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
