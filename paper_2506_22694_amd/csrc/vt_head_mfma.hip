// Draft step for many hidden rows (tree drafting, n > 8): the projection is a
// real GEMM  z[n, k] = h[n, d] W_trim[k, d]^T  and runs on the matrix cores
// (v_mfma_f32_16x16x32_bf16), still bound by the single pass over W_trim.
//
// One workgroup (8 waves) owns a tile of 128 rows of W_trim, 16 per wave:
//   * W is read from HBM exactly once, with row-contiguous 256-byte segments per
//     load instruction (4 rows x 256 B), several units in flight per wave; a unit
//     (16 rows x 128 columns) passes through a small wave-private LDS buffer that
//     re-lays it out as MFMA A-operands (row pitch 272 B: conflict-free reads);
//   * h is the B-operand: a chunk of KC columns of all hidden rows sits in LDS,
//     shared by the 8 waves, and is replaced chunk by chunk (h itself lives in L2);
//   * accumulators (16 W-rows x n hidden rows per wave) stay in registers over
//     the whole contraction; the logits are never written to memory;
//   * the tile's logits go to an LDS tile (aliasing the staging buffers) and the
//     same workgroup epilogue as the small-n kernel produces (max, sum-exp) and
//     the tile's best candidates per hidden row;
//   * a second small kernel merges the tiles: one wave per hidden row.
#include "vt_device.h"
#include "vt_launch.h"
#include "vt_step.h"
#include "vt_step_tail.h"
#include "vt_tree_dev.h"
#include <mutex>
#include <type_traits>

namespace vt {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kUnitCols = 128;                       // columns per staged unit (256 B per row)
constexpr int kStagePitch = 272;                     // bytes per staged row: 256 + 16 (bank spread)
constexpr int kStageUnitBytes = 16 * kStagePitch;    // one unit of one wave
constexpr int kStageBytes = kStepWaves * 2 * kStageUnitBytes;   // double-buffered, all waves of an 8-wave workgroup
constexpr int kPrefetchUnits = kMfmaPrefetchUnits;   // units of W in flight per wave (12 KiB)

__device__ __forceinline__ void stream_load16(u32x4 &dst, unsigned voff, const void *sbase) {
    asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(dst) : "v"(voff), "s"(sbase) : "memory");
}
// h pieces stay cacheable: every workgroup re-reads them from L2
__device__ __forceinline__ void cached_load16(u32x4 &dst, unsigned voff, const void *sbase) {
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(sbase) : "memory");
}
__device__ __forceinline__ void request_dword(int &dst, const int *p) {
    asm volatile("global_load_dword %0, %1, off" : "=v"(dst) : "v"(p) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_ids(int (&b)[11]) {
    asm volatile("s_waitcnt vmcnt(%11)"
                 : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7]),
                   "+v"(b[8]), "+v"(b[9]), "+v"(b[10])
                 : "n"(N));
}
constexpr int kMaxPieces = kMfmaChunkPieces;   // 16-byte pieces of an h chunk per thread
template <int N>
__device__ __forceinline__ void wait_pieces(u32x4 (&b)[kMaxPieces]) {
    asm volatile("s_waitcnt vmcnt(%9)"
                 : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7]),
                   "+v"(b[8])
                 : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_unit(u32x4 (&b)[4]) {
    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]) : "n"(N));
}

// MAXW: most waves a workgroup of this instantiation is launched with.  Eight is the rule: a wave per 16 rows of a
// 128-row tile.  Up to 8 hidden rows (NT = 1, all of h in LDS) the workgroup may have any number of waves up to
// MAXW = 12: the tile is then 16 * (waves / KS) rows, so that a head of any size up to 256 * 192 rows is cut into
// at most 256 tiles -- one round on 256 CUs -- instead of a second, nearly empty round of 128-row tiles.
// XG (eight waves, up to 8 hidden rows, d a multiple of 1024): the tile has 128 + extra_rows rows.  The rows past
// the 128th form one more 16-row group; wave w multiplies the w-th eighth of its columns after its own 16 rows, so
// all waves stream equal shares whatever the tile height is -- a head of k = 32975 rows is 256 tiles of 129 rows,
// one per CU, instead of 258 tiles of 128.  To keep a row's logit independent of the group it lies in, every logit is
// then formed from the partial sums P0 .. P7 of the eight column parts, each accumulated from zero in ascending
// order, as ((P0 + P1) + (P2 + P3)) + ((P4 + P5) + (P6 + P7)) -- in registers for a wave's own rows (two parts make
// one of the ranges described below), from LDS for the shared group.  All waves march over the columns of their
// own rows in step, as without the shared group.  (Measured alternatives at k = 32975, n = 8, d = 3072 / 4096:
// this kernel 40.1 / 54.0 us; every wave starting at another part, the eight partial sums kept in registers:
// 40.8 / 57.4; all rows cut into near-equal groups whose (group, part) tasks are dealt to the waves: 40.8 / 50.5;
// nine waves of 16 rows on 229 CUs: 41.4 / 51.4; the small-n kernel: 41.8 / 51.7.  The planner uses it where rows
// are not a multiple of 2 KiB.)
// XC != 0 (eight waves, more than 8 hidden rows -- h in LDS chunk by chunk, so the waves cannot split the columns
// between them while they march: all of them need the same chunk at the same time): the same tile of
// 128 + extra_rows rows.  Every logit of such a launch is formed from four column ranges, each accumulated from
// zero in ascending order, as (R0 + R1) + (R2 + R3) -- the order the rotated march below already uses where rows
// are a multiple of 2 KiB -- and the extra group passes the same range boundaries with the same instructions on
// the same operand layout: equal rows give equal logits.  Two ways to multiply the rows past the 128th:
// XC == 1 (two groups of hidden rows): the chunk of h in LDS is followed by the same columns of those rows, fetched
//   with it a chunk ahead; both operands of the extra group's products are then in LDS, in operand layout, and
//   multiplying them takes no place in any wave's W stream.  After its own units of chunk c wave (c + t) mod 8 does
//   that for hidden-row group t: 4 products per unit into an accumulator that lives in LDS between chunks, handed
//   from wave to wave at the chunk's barriers.
// XC == 2 (four groups): after the march, straight from global memory (their part of W is a few rows, h sits in
//   L2), one column range and two groups of hidden rows per wave, whole 256-byte row pieces turned into operand
//   layout through the wave's staging buffers.
// (Measured at k = 32975, d = 4096, n = 64 / n = 32, where k = 32768 takes 57 / 51.5 us and these tiles without
// the extra group's products 58.6 us at n = 64: 258 tiles of 128 rows 104 / 80.5 us; the extra group handed from
// wave to wave as more units of the W stream 79 / 61.9 -- the wave whose turn it is streams twice as many units
// as the others, who wait at the chunk's barrier; after the march 66 / 59.7, whatever its load pipeline (loads in
// matrix-core layout: 75; more units in flight, fewer operand rows loaded, a third staging buffer: 66.5 to 68.5) --
// every workgroup pulls all of h through its CU a second time, 134 MB at once over the L2s' 17 TB/s at n = 64;
// from LDS beside the chunk 69 / 56.5 -- with four groups of hidden rows the march is bound by its LDS traffic,
// to which the extra group adds a sixth, with two it is not.)
// MH: the tiles of several heads in one launch (see MultiHeadTable); one group of hidden rows, all of h in LDS.
template <int NT, int MAXW, bool XG = false, int XC = 0, bool MH = false>
__global__ void __launch_bounds__(MAXW *kWave) __attribute__((amdgpu_waves_per_eu(1, (MAXW + 3) / 4)))
head_mfma_kernel(const MfmaArgs a, const std::conditional_t<MH, MultiHeadTable, SingleHead> mh) {
    static_assert(!MH || (NT == 1 && !XG && XC == 0), "several heads per launch: one group of hidden rows, plain tiles");
    static_assert(!XG || (NT == 1 && MAXW == kStepWaves), "the shared row group is built for eight waves and one group of hidden rows");
    static_assert(XC == 0 || (!XG && MAXW == kStepWaves && ((XC == 1 && NT == 2) || (XC == 2 && NT == 4))),
                  "the extra row group in LDS is built for eight waves and two or four groups of hidden rows");
    constexpr bool XT = XG || XC != 0;      // tiles of 128 + extra_rows rows
    constexpr bool XL = XC == 1;            // the extra rows' columns in LDS beside the chunk of h
    constexpr bool XP = XC == 2;            // the extra rows in a pass after the march
    extern __shared__ __align__(16) unsigned char smem[];
    const int NW = MAXW == kStepWaves ? kStepWaves : a.nwaves;     // waves of this workgroup
    unsigned char *stage = smem;                       // [waves][2][16][272]
    unsigned char *hbuf = smem + (size_t)NW * 2 * kStageUnitBytes;   // [16 * NT or 8][hpitch]
    float *zt = reinterpret_cast<float *>(smem);       // logit tile, aliases both after the contraction

    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (a.ticket_clear != nullptr && blockIdx.x == 0 && threadIdx.x == 0)
        __hip_atomic_store(a.ticket_clear, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // Small heads (up to 8 hidden rows only): with fewer than ~160 tiles of 128 rows the tiles shrink to
    // 16 * NW / KS rows and KS waves share a group of 16 rows, each taking 1 / KS of the columns; their partial
    // logits meet in the LDS tile of the epilogue, summed in wave order.
    const int KS = NT == 1 ? a.ksplit : 1;
    const int tile_rows = 16 * (NW / KS) + (XT ? a.extra_rows : 0);
    const int rg = w / KS, ksi = w % KS;               // row group of the wave, its share of the columns
    // the head this tile belongs to, its first tile, size, rows and ids
    int hd = 0, tile_lo = 0, head_k = a.k;
    const void *head_W = a.W;
    const int *head_map = a.map;
    if constexpr (MH) {
        for (int q = 1; q < mh.n_heads; ++q) hd = (int)blockIdx.x >= mh.tile_first[q] ? q : hd;
        tile_lo = mh.tile_first[hd];
        head_k = mh.k[hd];
        head_W = mh.W[hd];
        head_map = mh.map[hd];
    }
    const int row0 = ((int)blockIdx.x - tile_lo) * tile_rows;
    const int rows_b = min(tile_rows, head_k - row0);
    const size_t rs = (size_t)a.d * 2;
    const int lrow = lane & 15, lgrp = lane >> 4;

    // per-lane byte offsets of the 4 load instructions of a unit: instruction j covers rows 4j..4j+3
    // of this wave's 16 rows, 16 lanes x 16 B per row; rows past the end of W repeat the last row
    unsigned voff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = min(16 * rg + 4 * j + lgrp, rows_b - 1);
        // (24-bit factors: a 64-bit multiply-add here may name a register with a load in flight as its unused half)
        voff[j] = __umul24((unsigned)r, (unsigned)(a.d * 2)) + (unsigned)lrow * 16u;
    }
    // the shared group: rows 128 .. of the tile (rows past its end repeat the last row)
    // (kept as the distance from the wave's own rows: choosing between two arrays by a run-time flag would put
    // both into scratch memory)
    unsigned vdelta[XT ? 4 : 1];
    if constexpr (XT) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = min(kMfmaTileRows + 4 * j + lgrp, rows_b - 1);
            vdelta[j] = __umul24((unsigned)r, (unsigned)(a.d * 2)) + (unsigned)lrow * 16u - voff[j];
        }
    }
    const char *Wt = static_cast<const char *>(head_W) + (size_t)row0 * rs;
    const int nunits = a.d / kUnitCols;
    const int nun = nunits / KS;                       // units of this wave's own rows
    const int PL = nunits / 8;                         // XG: units per column part
    const int ntot = XG ? nun + PL : nun;              // units this wave streams
    // Every workgroup marches over the columns of its 128 rows; if all of them sat in the same column
    // stripe of W at the same time (rows are d * 2 bytes apart) the requests would crowd a subset of the
    // HBM channels (measured: 5.7 instead of 6.7 TB/s).  So the contraction is cut into four column ranges
    // and workgroup b starts with range (b / 8) % 4 -- b % 8 is the XCD -- and wraps around.  Each range
    // R0..R3 is accumulated from zero in ascending order and the logit is (R0 + R1) + (R2 + R3); float
    // addition commutes, so that value does not depend on where the workgroup started (equal rows of W
    // give equal logits in whichever tile they lie).  Two sets of registers hold the finished ranges:
    // ranges finish in the order rot, rot + 1, .. and the k-th to finish is added to set
    // {0, 0, 1, 1}[k] for an even start, {0, 1, 1, 0}[k] for an odd one, which pairs R0 with R1 and R2 with R3.
    // (Rows a multiple of 4 KiB apart are the ones that crowd; at d = 3072 the plain march is 0.6 us faster.)
    // (XC: the four ranges at any row length, the start rotated as everywhere only where it pays)
    const bool rotate = KS == 1 && nunits >= 8 && (XC != 0 || a.d % 2048 == 0);
    const int rot = (rotate && a.d % 2048 == 0) ? ((int)blockIdx.x >> 3) & 3 : 0;
    // first units of ranges 1..3.  When a quarter of a row is itself a multiple of 4 KiB (d = 8192) quarter starts
    // would crowd the same channels again: the boundaries are skewed by 1, 2 and 3 KiB (any fixed partition of the
    // columns keeps the rounding independent of the start)
    const int skew = ((nunits / 4) * kUnitCols * 2) % 4096 == 0 ? 4 : 0;
    const int rb1 = nunits / 4 + skew, rb2 = nunits / 2 + 2 * skew, rb3 = (3 * nunits) / 4 + 3 * skew;
    const int ustart = KS > 1 ? ksi * nun : rot == 0 ? 0 : rot == 1 ? rb1 : rot == 2 ? rb2 : rb3;
    const int hstart = KS > 1 ? 0 : ustart;            // first unit of h's layout in LDS (the same for all waves)
    // unit processed at step s (0 <= s < nun)
    auto unit_of = [&](int s) {
        const int u = ustart + s;
        return u >= nunits ? u - nunits : u;
    };
    auto load_unit = [&](int u, u32x4(&dst)[4]) {
        if constexpr (XG) {
            u = min(u, ntot - 1);
            const bool own = u < nun;
            const char *p = Wt + (size_t)(own ? unit_of(u) : w * PL + (u - nun)) * (kUnitCols * 2);
            const unsigned shared = own ? 0u : 0xFFFFFFFFu;
#pragma unroll
            for (int j = 0; j < 4; ++j) stream_load16(dst[j], voff[j] + (vdelta[j] & shared), p);
        } else {
            const char *p = Wt + (size_t)unit_of(min(u, nun - 1)) * (kUnitCols * 2);
#pragma unroll
            for (int j = 0; j < 4; ++j) stream_load16(dst[j], voff[j], p);
        }
    };
    u32x4 areg[kPrefetchUnits][4];

    f32x4 acc[NT];
    f32x4 pair0[NT], pair1[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = pair0[t] = pair1[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    int closed = 0;        // ranges finished so far
#define VT_CLOSE_RANGE()                                                              \
    {                                                                                 \
        const bool to1 = (rot & 1) ? (closed == 1 || closed == 2) : closed >= 2;      \
        _Pragma("unroll") for (int t = 0; t < NT; ++t) {                              \
            const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};                             \
            pair0[t] += to1 ? zero : acc[t];      /* adding zero changes nothing */   \
            pair1[t] += to1 ? acc[t] : zero;                                          \
            acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};                                       \
        }                                                                             \
        ++closed;                                                                     \
    }
    // XG: a range is two column parts.  The first of them waits in `stash`; when the second is complete their sum
    // goes the way of a range above.  (Ranges start at even parts, so the parts of a range follow one another.)
    f32x4 stash = f32x4{0.f, 0.f, 0.f, 0.f};
    int pcount = 0;        // units of the current part done so far
    bool second = false;   // the current part is the second of its range
    auto close_part = [&]() {
        if (!second) {
            stash = acc[0];
            acc[0] = f32x4{0.f, 0.f, 0.f, 0.f};
        } else {
            acc[0] = stash + acc[0];
            VT_CLOSE_RANGE()
        }
        second = !second;
        pcount = 0;
    };

    unsigned char *my_stage = stage + (size_t)w * 2 * kStageUnitBytes;
    // staging writes: instruction j, lane (row 4j + lgrp, 16-byte chunk lrow)
    // operand reads : lane (row lrow, k-group lgrp) of k-step ks -> bytes ks*64 + lgrp*16
    const int wr_off = lgrp * kStagePitch + lrow * 16;
    const int rd_off = lrow * kStagePitch + lgrp * 16;
    // up to 8 hidden rows: LDS holds 8 rows of h and lanes 8..15 of the operand repeat them (their products
    // are never read)
    const int hrows = a.n <= 8 ? 8 : 16 * NT;
    const int hrow_off = (lrow & (hrows - 1)) * a.hpitch + lgrp * 16;

    // ---- h chunks: the columns of KC / 128 consecutive steps, of every hidden row (zero rows up to 16 * NT), live in LDS.  The next
    // chunk is fetched into registers while the current one is consumed, so its L2 latency is hidden;
    // two barriers per chunk swap it in.
    const int units_per_chunk = a.KC / kUnitCols;
    const int nchunks = (a.d + a.KC - 1) / a.KC;
    u32x4 hp[kMaxPieces];
    // piece e = q * 512 + tid of a chunk is (hidden row e / ppr, 16-byte piece e % ppr); one division per
    // chunk, then a carry per step
    // XC == 1: the pieces of h are followed, from a piece number of their own on, by those of the 16 extra rows (the same
    // columns of W; rows past the tile's end repeat its last row), which land in LDS rows 16 NT .. behind h.
    auto fetch_chunk = [&](int c) {
        const int c0 = c * a.KC;
        const int ppr = min(a.KC, a.d - c0) >> 3;        // pieces per row
        const int step_r = (NW * kWave) / ppr, step_p = (NW * kWave) % ppr;
        const int r_first = (int)threadIdx.x / ppr, pc_first = (int)threadIdx.x % ppr;
        int r = r_first, pc = pc_first;
        const int qx = XL ? (16 * NT * ppr + NW * kWave - 1) / (NW * kWave) : kMaxPieces;      // first piece of the extra rows
        const int s0 = c * (a.KC / kUnitCols);           // first step of the chunk
        const char *hbase = static_cast<const char *>(a.h);
#pragma unroll
        for (int q = 0; q < kMaxPieces; ++q) {
            hp[q] = u32x4{0u, 0u, 0u, 0u};
            const bool extra = XL && q >= qx;            // (uniform)
            if (XL && q == qx) {
                r = r_first;
                pc = pc_first;
            }
            // 16 pieces per unit: piece pc belongs to step s0 + pc / 16
            int ua = hstart + s0 + (pc >> 4);
            ua = ua >= nunits ? ua - nunits : ua;
            // few hidden rows may be picked out of a larger batch (their indices are packed in row_pack)
            const int hr = extra ? min(kMfmaTileRows + r, rows_b - 1)
                                 : a.indexed ? (int)((a.row_pack >> (8 * (r & 7))) & 0xFFull) : r;
            const unsigned off = __umul24((unsigned)hr, (unsigned)(a.d * 2)) + (unsigned)ua * (kUnitCols * 2) + (unsigned)(pc & 15) * 16u;
            if (r < (extra ? 16 : a.n)) cached_load16(hp[q], off, extra ? static_cast<const void *>(Wt) : static_cast<const void *>(hbase));
            r += step_r;
            pc += step_p;
            if (pc >= ppr) {
                pc -= ppr;
                ++r;
            }
        }
    };
    auto store_chunk = [&](int c) {
        const int ppr = min(a.KC, a.d - c * a.KC) >> 3;
        const int step_r = (NW * kWave) / ppr, step_p = (NW * kWave) % ppr;
        const int r_first = (int)threadIdx.x / ppr, pc_first = (int)threadIdx.x % ppr;
        int r = r_first, pc = pc_first;
        const int qx = XL ? (16 * NT * ppr + NW * kWave - 1) / (NW * kWave) : kMaxPieces;
#pragma unroll
        for (int q = 0; q < kMaxPieces; ++q) {
            const bool extra = XL && q >= qx;
            if (XL && q == qx) {
                r = r_first;
                pc = pc_first;
            }
            if (r < (extra ? 16 : hrows))
                *reinterpret_cast<u32x4 *>(hbuf + (size_t)(extra ? 16 * NT + r : r) * a.hpitch + pc * 16) = hp[q];
            r += step_r;
            pc += step_p;
            if (pc >= ppr) {
                pc -= ppr;
                ++r;
            }
        }
    };
    // Target ids of the tile rows this lane ranks in the epilogue (two layouts, see below).  They are requested
    // by hand like everything else here and first of all: a load the compiler knows of would get a wait from
    // it wherever it sees fit, and since loads return in order any such wait also waits for the W prefetch.
    // (ids[2 ..]: rows lrow + 16 q for the four-rows-per-pass epilogue of more than 8 hidden rows; with up to
    // 12 waves or a shared row group -- up to 8 hidden rows, a wave per row -- ids[2] is the row lane + 128 of a tile
    // of up to 192 rows)
    // (With four groups of hidden rows and the handed-on extra rows there are no registers to spare for them during
    // the contraction: that variant reads them afterwards.)
    constexpr bool IDS_LATE = XC != 0 && NT == 4;
    int ids[11];
    if constexpr (!IDS_LATE) {
        request_dword(ids[0], head_map + row0 + min(lane, rows_b - 1));
        request_dword(ids[1], head_map + row0 + min(lane + kWave, rows_b - 1));
#pragma unroll
        for (int q = 0; q < 9; ++q)
            request_dword(ids[2 + q],
                          head_map + row0 + min((MAXW > kStepWaves || XG) ? lane + 2 * kWave : lrow + 16 * q, rows_b - 1));
    }
    fetch_chunk(0);                       // everything waits for it
#pragma unroll
    for (int x = 0; x < kPrefetchUnits; ++x) {
        load_unit(x, areg[x]);
    }
    wait_pieces<4 * kPrefetchUnits>(hp);  // the W prefetch stays in flight
    if constexpr (!IDS_LATE) wait_ids<4 * kPrefetchUnits>(ids);    // older than the chunk: they have landed too
    store_chunk(0);
    __syncthreads();
    int id0 = 0, id1 = 0;
    int idq[9];
    if constexpr (!IDS_LATE) {
        id0 = ids[0];
        id1 = ids[1];
#pragma unroll
        for (int q = 0; q < 9; ++q) idq[q] = ids[2 + q];
    }


    // Units are consumed in order; unit u sits in register slot u % kPrefetchUnits.  Between a hand-issued
    // load and its wait the compiler believes the registers already hold their data, so the order of loads
    // and waits must be the same on every path through the code, not only on those that the values of
    // u and c allow: the loop is written so that its shape alone guarantees it (a build step follows every
    // path of the compiled kernel and checks this).
    int u = 0;
    auto run_unit = [&](u32x4(&ar)[4], int uc) {
        // unit u's four loads are the oldest outstanding of the W stream
        wait_unit<4 * (kPrefetchUnits - 1)>(ar);
        unsigned char *sb = my_stage + (u & 1) * kStageUnitBytes;
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(sb + 4 * j * kStagePitch + wr_off) = ar[j];
        load_unit(u + kPrefetchUnits, ar);
        const unsigned char *hb = hbuf + hrow_off + (size_t)uc * (kUnitCols * 2);
        if constexpr (XG) {
            if (pcount == PL) close_part();      // (at u == nun this closes the last part of the wave's own rows)
            if (u == nun) {
                // own rows complete: their logits wait in pair0; the shared group's part starts from zero
                pair0[0] = pair0[0] + pair1[0];
            }
            if (u >= nun) {
                // the shared group's unit w PL + (u - nun): where it lies in h's (rotated) layout in LDS
                int pos = w * PL + (u - nun) - hstart;
                pos = pos < 0 ? pos + nunits : pos;
                hb = hbuf + hrow_off + (size_t)pos * (kUnitCols * 2);
            }
            ++pcount;
        } else if (rotate && u > 0) {
            const int ua = unit_of(u);
            if (ua == 0 || ua == rb1 || ua == rb2 || ua == rb3) VT_CLOSE_RANGE()
        }
        // operands of two k-steps are read before their MFMAs are issued, so that the LDS latency is paid
        // once per pair and not once per MFMA
#pragma unroll
        for (int kp = 0; kp < 4; kp += 2) {
            u32x4 av[2], bv[2][NT];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                av[ks] = *reinterpret_cast<const u32x4 *>(sb + rd_off + (kp + ks) * 64);
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    bv[ks][t] = *reinterpret_cast<const u32x4 *>(hb + (size_t)t * 16 * a.hpitch + (kp + ks) * 64);
            }
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av[ks]),
                                                                     __builtin_bit_cast(bf16x8, bv[ks][t]), acc[t],
                                                                     0, 0, 0);
            }
        }
        ++u;
    };
    // Chunks that have a successor hold a multiple of kPrefetchUnits units (the host plans them so): the
    // next chunk is requested, whole rounds of units run without any test in between, and by then every
    // piece of the next chunk has 4 * kPrefetchUnits younger loads behind it.
    // XC == 1: the extra group's accumulators live in LDS behind the chunk, [acc, pair0, pair1][hidden-row group][lane],
    // and start at zero (the wave that has a group in the first chunk sets them).  extra_group(t, ..) multiplies the
    // chunk's `count` units (march positions u_first ..) of the extra rows by hidden-row group t: the same operand
    // layout, instructions and range boundaries as a wave's own rows in run_unit; t only selects LDS addresses.
    f32x4 *xs = reinterpret_cast<f32x4 *>(smem + a.xoff);
    auto extra_group = [&](int t, int count, int u_first, int xclosed, bool first, bool last) {
        f32x4 *sacc = xs + (size_t)(0 * NT + t) * kWave + lane;
        f32x4 *spair0 = xs + (size_t)(1 * NT + t) * kWave + lane;
        f32x4 *spair1 = xs + (size_t)(2 * NT + t) * kWave + lane;
        if (first) *sacc = *spair0 = *spair1 = f32x4{0.f, 0.f, 0.f, 0.f};
        f32x4 xa = *sacc;
        const unsigned char *arow = hbuf + (size_t)(16 * NT + lrow) * a.hpitch + lgrp * 16;
        const unsigned char *brow = hbuf + (size_t)(16 * t + lrow) * a.hpitch + lgrp * 16;
        auto close = [&]() {
            const bool to1 = (rot & 1) ? (xclosed == 1 || xclosed == 2) : xclosed >= 2;
            f32x4 *dst = to1 ? spair1 : spair0;
            *dst = *dst + xa;
            xa = f32x4{0.f, 0.f, 0.f, 0.f};
            ++xclosed;
        };
        // (a unit's h operands are on their way from LDS while the unit before it is multiplied)
        u32x4 bv[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) bv[ks] = *reinterpret_cast<const u32x4 *>(brow + ks * 64);
        for (int j = 0; j < count; ++j) {
            u32x4 av[4], bn[4];
            const size_t jn = (size_t)min(j + 1, count - 1) * (kUnitCols * 2);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                av[ks] = *reinterpret_cast<const u32x4 *>(arow + (size_t)j * (kUnitCols * 2) + ks * 64);
                bn[ks] = *reinterpret_cast<const u32x4 *>(brow + jn + ks * 64);
            }
            const int xu = u_first + j;
            if (xu > 0) {
                const int ua = unit_of(xu);
                if (ua == 0 || ua == rb1 || ua == rb2 || ua == rb3) close();
            }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                xa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av[ks]),
                                                             __builtin_bit_cast(bf16x8, bv[ks]), xa, 0, 0, 0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bv[ks] = bn[ks];
        }
        if (last) {
            close();
            xa = *spair0 + *spair1;
        }
        *sacc = xa;
    };
    for (int c = 0; c + 1 < nchunks; ++c) {
        fetch_chunk(c + 1);
        const int u_first = u, closed_first = closed;
        int uc = 0;
        do {
#pragma unroll
            for (int x = 0; x < kPrefetchUnits; ++x) run_unit(areg[x], uc++);
        } while (uc < units_per_chunk);
        if constexpr (XL) {
            const int t = (w - c) & 7;
            if (t < NT) extra_group(t, units_per_chunk, u_first, closed_first, c == 0, false);
        }
        wait_pieces<4 * kPrefetchUnits>(hp);
        __syncthreads();       // every wave is done with the current chunk
        store_chunk(c + 1);
        __syncthreads();
    }
    // the last chunk: any number of units -- whole rounds, then the one or two that remain
    {
        const int u_first = u, closed_first = closed;
        int uc = KS > 1 ? ustart : 0;      // position of the wave's first unit in h's LDS layout
        for (int rounds = (ntot - u) / kPrefetchUnits; rounds > 0; --rounds) {
#pragma unroll
            for (int x = 0; x < kPrefetchUnits; ++x) run_unit(areg[x], uc++);
        }
        static_assert(kPrefetchUnits == 3, "the remainder below is written for rounds of three");
        if (u < ntot) {
            run_unit(areg[0], uc++);
            if (u < ntot) run_unit(areg[1], uc++);
        }
        if constexpr (XL) {
            const int t = (w - (nchunks - 1)) & 7;
            if (t < NT) extra_group(t, ntot - u_first, u_first, closed_first, nchunks == 1, true);
        }
    }
    // prefetches past the last unit are still in flight: let them land before their registers die
#pragma unroll
    for (int x = 0; x < kPrefetchUnits; ++x) wait_unit<0>(areg[x]);
    // XC == 2: the extra rows.  Wave w takes column range w % 4 and the groups of hidden rows w / 4 (+ 2), and repeats on
    // them what the march did on its own rows: the same instructions in the same order on the same operand layout.
    // Nothing hand-issued is in flight any more, so these are ordinary loads: whole 256-byte row pieces of W and,
    // this time, of h as well (it is in L2; the chunk in LDS is long gone), both turned into operand layout
    // through the wave's own staging buffers, XUB units per round trip.
    constexpr int XGROUPS = XP ? NT / 2 : 1;
    constexpr int XUB = NT == 2 ? 4 : 2;
    f32x4 xacc[XGROUPS];
    if constexpr (XP) {
        const int q = w & 3;
        const int ub = q == 0 ? 0 : q == 1 ? rb1 : q == 2 ? rb2 : rb3;
        const int ue = q == 0 ? rb1 : q == 1 ? rb2 : q == 2 ? rb3 : nunits;
        // (hidden rows past n repeat row n - 1: their columns of the result are never read)
        unsigned boff[XGROUPS][4];
        const char *hbase = static_cast<const char *>(a.h);
#pragma unroll
        for (int g = 0; g < XGROUPS; ++g) {
            xacc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j)
                boff[g][j] = __umul24((unsigned)min(16 * ((w >> 2) + 2 * g) + 4 * j + lgrp, a.n - 1), (unsigned)(a.d * 2)) +
                             (unsigned)lrow * 16u;
        }
        unsigned char *sa = my_stage, *sb = my_stage + kStageUnitBytes;
        for (int u0 = ub; u0 < ue; u0 += XUB) {
            u32x4 ar[XUB][4], br[XUB][XGROUPS][4];
#pragma unroll
            for (int x = 0; x < XUB; ++x) {
                const size_t col = (size_t)min(u0 + x, ue - 1) * (kUnitCols * 2);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    ar[x][j] = *reinterpret_cast<const u32x4 *>(Wt + col + (voff[j] + vdelta[j]));
#pragma unroll
                    for (int g = 0; g < XGROUPS; ++g)
                        br[x][g][j] = *reinterpret_cast<const u32x4 *>(hbase + col + boff[g][j]);
                }
            }
#pragma unroll
            for (int x = 0; x < XUB; ++x) {
                if (u0 + x < ue) {
                    u32x4 av[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(sa + 4 * j * kStagePitch + wr_off) = ar[x][j];
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) av[ks] = *reinterpret_cast<const u32x4 *>(sa + rd_off + ks * 64);
#pragma unroll
                    for (int g = 0; g < XGROUPS; ++g) {
                        u32x4 bv[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            *reinterpret_cast<u32x4 *>(sb + 4 * j * kStagePitch + wr_off) = br[x][g][j];
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks) bv[ks] = *reinterpret_cast<const u32x4 *>(sb + rd_off + ks * 64);
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks)
                            xacc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av[ks]),
                                                                              __builtin_bit_cast(bf16x8, bv[ks]),
                                                                              xacc[g], 0, 0, 0);
                    }
                }
            }
        }
    }
    if constexpr (IDS_LATE) {
        id0 = head_map[row0 + min(lane, rows_b - 1)];
        id1 = head_map[row0 + min(lane + kWave, rows_b - 1)];
#pragma unroll
        for (int q = 0; q < 9; ++q) idq[q] = head_map[row0 + min(lrow + 16 * q, rows_b - 1)];
    }

    if constexpr (XG) {
        // acc[0]: the shared group's partial logits over this wave's column part; pair0[0]: the own rows' logits
    } else if (rotate) {
        VT_CLOSE_RANGE()
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = pair0[t] + pair1[t];
    }
#undef VT_CLOSE_RANGE

    // ---- logits of this tile -> LDS tile zt[i][t] (aliases staging and h)
    __syncthreads();
    const int tp = (XT ? kMfmaTileRows + 16 : MAXW == kStepWaves ? kMfmaTileRows : tile_rows) + 1;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int i = 16 * t + lrow;       // hidden row of this lane
        if (i < a.n) {
            float *dst = zt + ((size_t)ksi * a.n + i) * tp + 16 * rg + 4 * lgrp;      // partial ksi of row i
            const f32x4 v = XG ? pair0[t] : acc[t];
            dst[0] = v.x;
            dst[1] = v.y;
            dst[2] = v.z;
            dst[3] = v.w;
        }
    }
    if constexpr (XL) {
        // the extra rows' logits wait in LDS (behind the chunk, not under the tile) in accumulator layout: wave t
        // copies those of hidden rows 16 t ..
        if (w < NT) {
            const f32x4 v = xs[(size_t)w * kWave + lane];
            const int i = 16 * w + lrow;
            if (i < a.n) {
                float *dst = zt + (size_t)i * tp + kMfmaTileRows + 4 * lgrp;
                dst[0] = v.x;
                dst[1] = v.y;
                dst[2] = v.z;
                dst[3] = v.w;
            }
        }
    }
    if constexpr (XP) {
        // the extra rows: the range sums xq[range][hidden row][16] behind the tile and its candidate keys, then the
        // same two levels of additions as in the registers of the own rows
        float *xq = reinterpret_cast<float *>(smem + (((size_t)a.n * tp * sizeof(float) + 15) & ~(size_t)15) +
                                              kStepWaves * 4 * 16 * sizeof(unsigned long long));
#pragma unroll
        for (int g = 0; g < XGROUPS; ++g) {
            const int i = 16 * ((w >> 2) + 2 * g) + lrow;
            if (i < a.n) {
                float *dst = xq + ((size_t)(w & 3) * a.n + i) * 16 + 4 * lgrp;
                dst[0] = xacc[g].x;
                dst[1] = xacc[g].y;
                dst[2] = xacc[g].z;
                dst[3] = xacc[g].w;
            }
        }
        __syncthreads();
        const size_t ps = (size_t)a.n * 16;      // from one range to the next
        for (int e = (int)threadIdx.x; e < 16 * a.n; e += kStepWaves * kWave) {
            const float *x = xq + e;
            zt[(size_t)(e >> 4) * tp + kMfmaTileRows + (e & 15)] = (x[0] + x[ps]) + (x[2 * ps] + x[3 * ps]);
        }
    }
    if constexpr (XG) {
        // the shared group: the eight waves' partials xq[part][hidden row][16] behind the tile and its candidate
        // keys, then the same tree as in the registers above
        float *xq = reinterpret_cast<float *>(smem + 8192 + kStepWaves * 3 * kWave * sizeof(unsigned long long));
        if (lrow < a.n) {
            float *dst = xq + ((size_t)w * a.n + lrow) * 16 + 4 * lgrp;
            dst[0] = acc[0].x;
            dst[1] = acc[0].y;
            dst[2] = acc[0].z;
            dst[3] = acc[0].w;
        }
        __syncthreads();
        const int e = (int)threadIdx.x;
        if (e < 16 * a.n) {
            const int i = e >> 4, r = e & 15;
            const float *x = xq + (size_t)i * 16 + r;
            const size_t ps = (size_t)a.n * 16;      // from one part to the next
            const float s01 = x[0] + x[ps], s23 = x[2 * ps] + x[3 * ps];
            const float s45 = x[4 * ps] + x[5 * ps], s67 = x[6 * ps] + x[7 * ps];
            zt[(size_t)i * tp + kMfmaTileRows + r] = (s01 + s23) + (s45 + s67);
        }
    }
    __syncthreads();

    if (a.zbuf != nullptr) {
        // store-only tail: the tile's logits go to z [n, k]; a workgroup per hidden row finishes the step
        // (row_select_kernel).  One wave copies a hidden row's 128 logits (512 contiguous bytes) at a time.
        for (int i = w; i < a.n; i += NW) {
            const float *src = zt + (size_t)i * tp;
            float *dst = a.zbuf + (size_t)i * a.k + row0;
            for (int t = lane; t < rows_b; t += kWave) dst[t] = src[t];
        }
        return;
    }

    if (a.L <= 16 && a.n > kStepWaves) {
        // four hidden rows per wave and pass (16 lanes each)
        // candidate keys of the threshold selection: 4 rows x 16 keys per wave, behind the logit tile
        unsigned long long *cand4 =
            reinterpret_cast<unsigned long long *>(smem + (((size_t)a.n * tp * sizeof(float) + 15) & ~(size_t)15)) +
            (size_t)w * 4 * 16;
        for (int i0 = 4 * w; i0 < a.n; i0 += 4 * NW) {
            if constexpr (XC != 0) {
                block_epilogue_rows4<9>(zt, tp, i0, a.n, rows_b, a.L, idq, a.out_logp_full, (size_t)a.k, row0, a.pms,
                                        a.pkeys, a.nlists, (int)blockIdx.x, lane, cand4);
            } else {
                const int idq8[8] = {idq[0], idq[1], idq[2], idq[3], idq[4], idq[5], idq[6], idq[7]};
                block_epilogue_rows4<8>(zt, tp, i0, a.n, rows_b, a.L, idq8, a.out_logp_full, (size_t)a.k, row0, a.pms,
                                        a.pkeys, a.nlists, (int)blockIdx.x, lane, cand4);
            }
        }
    } else {
        // a wave per hidden row (all of them at once for n <= 8); candidate keys of the threshold selection
        // sit behind the logit tile, 1 KiB per wave
        const size_t ztile = ((size_t)KS * a.n * tp * sizeof(float) + 15) & ~(size_t)15;
        constexpr int kCandPerWave = (MAXW > kStepWaves || XG) ? 3 * kWave : 2 * kWave;      // one key per tile row
        unsigned long long *cand =
            a.n <= kStepWaves
                ? reinterpret_cast<unsigned long long *>(smem + (ztile > 8192 ? ztile : 8192)) + (size_t)w * kCandPerWave
                : nullptr;
        for (int i = w; i < a.n; i += NW) {
            const float *zrow = zt + (size_t)i * tp;
            float *full = a.out_logp_full ? a.out_logp_full + (size_t)i * a.k + row0 : nullptr;
            unsigned long long *pms_slot = a.pms + (size_t)i * a.nlists + blockIdx.x;
            unsigned long long *pk_slot = a.pkeys + ((size_t)i * a.nlists + blockIdx.x) * a.L;
            if constexpr (MH) {
                // a hidden row of another head: nothing of this tile is its business -- an empty list, and a
                // (max, sum-exp) pair that adds nothing to any log-sum-exp
                if ((int)((mh.head_of_row >> (8 * i)) & 0xFFull) != hd) {
                    if (lane == 0) publish_u64(pms_slot, (unsigned long long)__float_as_uint(-3.0e38f));
                    if (lane < a.L) publish_u64(pk_slot + lane, kNoKey);
                    continue;
                }
            }
            // the logit is the sum of the KS partial tiles, in wave order
            if constexpr (MAXW > kStepWaves || XG) {
                const int idq3[3] = {id0, id1, idq[0]};
                block_epilogue_core<3>(zrow, KS, a.n * tp, rows_b, a.L, idq3, full, pms_slot, pk_slot, lane, cand);
            } else {
                block_epilogue_small(zrow, KS, a.n * tp, rows_b, a.L, id0, id1, full, pms_slot, pk_slot, lane, cand);
            }
        }
    }
}

// Re-lays h so that one B-operand load of the kernel below is 1 KiB of consecutive bytes: piece
// (unit u, k-step ks, 16-row group g, lane) holds the 8 columns 128 u + 32 ks + 8 (lane / 16) .. of
// hidden row 16 g + lane % 16 (rows past n repeat row n - 1; their products are never read).
// Read in place, hidden rows lie d * 2 bytes apart and a load touches 16 of them, which the L2
// serves at a fraction of the rate of consecutive lines.
__global__ void __launch_bounds__(256) pack_h_kernel(const u32x4 *__restrict__ h, u32x4 *__restrict__ hp, int n,
                                                     int d, int groups, long long pieces) {
    const long long x = (long long)blockIdx.x * 256 + threadIdx.x;
    if (x >= pieces) return;
    const int lane = (int)(x & 63);
    const long long y = x >> 6;
    const int g = (int)(y % groups);
    const long long z = y / groups;          // 4 u + ks
    const int i = min(16 * g + (lane & 15), n - 1);
    const long long col16 = z * 4 + (lane >> 4);   // 16-byte column piece of the row
    hp[x] = h[(long long)i * (d / 8) + col16];
}

// ------------------------------------------------------------------ many hidden rows (n > 64)
// With hundreds of hidden rows a chunk of h no longer fits LDS next to anything else, so the
// roles are swapped: the unit of W (128 rows x 128 columns, loaded by the 8 waves as above, 16
// rows each) is staged in LDS *shared* by the workgroup, double-buffered with one barrier per
// unit, and every wave owns 16 * NTW hidden rows whose B-operands come straight from h (L2) into
// registers, one unit ahead.  A wave multiplies all 128 rows of the tile (8 M-tiles) by its
// hidden rows.
template <int N, int CNT>
__device__ __forceinline__ void wait_regs(u32x4 (&b)[CNT]) {
    static_assert(CNT == 4 || CNT == 8, "register group size");
    if constexpr (CNT == 4) {
        asm volatile("s_waitcnt vmcnt(%4)" : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]) : "n"(N));
    } else {
        asm volatile("s_waitcnt vmcnt(%8)"
                     : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7])
                     : "n"(N));
    }
}

template <int NTW>
__global__ void __launch_bounds__(kStepWaves *kWave) head_mfma_wide_kernel(const MfmaArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int kUbufBytes = kMfmaTileRows * kStagePitch;   // one staged unit of the whole tile
    float *zt = reinterpret_cast<float *>(smem);                // logit tile, aliases the unit buffers afterwards
    constexpr int PU = kPrefetchUnits;
    constexpr int NB = 4 * NTW;                                  // B-operand loads per unit

    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (a.ticket_clear != nullptr && blockIdx.x == 0 && threadIdx.x == 0)
        __hip_atomic_store(a.ticket_clear, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int row0 = blockIdx.x * kMfmaTileRows;
    const int rows_b = min(kMfmaTileRows, a.k - row0);
    const size_t rs = (size_t)a.d * 2;
    const int lrow = lane & 15, lgrp = lane >> 4;
    const int nunits = a.d / kUnitCols;

    // W: this wave loads rows 16w .. 16w+15 of the tile, 4 rows x 256 B per instruction
    unsigned voff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = min(16 * w + 4 * j + lgrp, rows_b - 1);
        voff[j] = (unsigned)((size_t)r * rs + (size_t)lrow * 16);
    }
    const unsigned voff_dummy = (unsigned)lane * 16;
    const char *Wt = static_cast<const char *>(a.W) + (size_t)row0 * rs;
    // Rotated start of the column march, as in head_mfma_kernel (same ranges, same pairing of the partial
    // sums), for up to 128 hidden rows.  With more, the accumulators leave no registers for the pairs, and
    // the workgroups' B-operands would come from four regions of h at once, which the L2 serves more slowly
    // than the crowding costs (measured).
    const bool rotate = NTW == 1 && nunits >= 8 && a.d % 2048 == 0;
    const int rot = rotate ? ((int)blockIdx.x >> 3) & 3 : 0;
    const int skew = ((nunits / 4) * kUnitCols * 2) % 4096 == 0 ? 4 : 0;      // as in head_mfma_kernel
    const int rb1 = nunits / 4 + skew, rb2 = nunits / 2 + 2 * skew, rb3 = (3 * nunits) / 4 + 3 * skew;
    const int ustart = rot == 0 ? 0 : rot == 1 ? rb1 : rot == 2 ? rb2 : rb3;
    auto unit_of = [&](int s) {       // unit processed at step s < nunits
        const int u = ustart + s;
        return u >= nunits ? u - nunits : u;
    };
    // past the last unit the pipeline keeps its shape by reading the start of h (L2, in bounds)
    auto load_unit = [&](int u, u32x4(&dst)[4]) {
        const bool real = u < nunits;
        const char *p = real ? Wt + (size_t)unit_of(u) * (kUnitCols * 2) : static_cast<const char *>(a.h);
#pragma unroll
        for (int j = 0; j < 4; ++j) stream_load16(dst[j], real ? voff[j] : voff_dummy, p);
    };
    // h: B-operands of hidden rows 16 * (NTW * w + t) + lrow, k-group lgrp, four k-steps per unit,
    // from the re-laid copy: 1 KiB per (unit, k-step, 16-row group)
    const char *hpk = static_cast<const char *>(a.hpack) + (size_t)(NTW * w) * 1024;
    auto load_b = [&](int u, u32x4(&dst)[NB]) {
        const char *p = hpk + (size_t)unit_of(min(u, nunits - 1)) * (4 * 8 * NTW * 1024);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
            for (int t = 0; t < NTW; ++t) cached_load16(dst[ks * NTW + t], voff_dummy, p + (ks * 8 * NTW + t) * 1024);
        }
    };

    u32x4 areg[PU][4];
    u32x4 breg[2][NB];
    f32x4 acc[8][NTW];
    constexpr int NPAIR = NTW == 1 ? 8 : 1;      // pair accumulators exist only where the start rotates
    f32x4 pair0[NPAIR], pair1[NPAIR];
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
#pragma unroll
        for (int t = 0; t < NTW; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int mt = 0; mt < NPAIR; ++mt) pair0[mt] = pair1[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    int closed = 0;        // ranges finished so far
    auto close_range = [&]() {
        if constexpr (NTW == 1) {
            // always into pair0; the two sets trade places when the next range belongs to the other pair
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) {
                pair0[mt] += acc[mt][0];
                acc[mt][0] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            const bool trade = (rot & 1) ? (closed == 0 || closed == 2) : closed == 1;
            if (trade) {
#pragma unroll
                for (int mt = 0; mt < 8; ++mt) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {      // in place: no temporaries
                        float x = pair0[mt][c], y = pair1[mt][c];
                        asm volatile("v_swap_b32 %0, %1" : "+v"(x), "+v"(y));
                        pair0[mt][c] = x;
                        pair1[mt][c] = y;
                    }
                }
            }
            ++closed;
        }
    };
    const int wr_off = (16 * w + lgrp) * kStagePitch + lrow * 16;   // + 4 j rows
    const int rd_off = lrow * kStagePitch + lgrp * 16;              // + 16 mt rows, + ks * 64

    // ---- prologue: units 0 .. PU-1 and B(0) requested; unit 0 staged
#pragma unroll
    for (int x = 0; x < PU; ++x) load_unit(x, areg[x]);
    load_b(0, breg[0]);
    wait_regs<0, 4>(areg[0]);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        *reinterpret_cast<u32x4 *>(smem + 4 * j * kStagePitch + wr_off) = areg[0][j];
    load_unit(PU, areg[0]);
    __syncthreads();
    // target ids of the tile rows this lane ranks in the epilogue (two layouts).  With two hidden-row
    // groups per wave they are requested after the contraction, which has no registers to spare for them.
    int id0 = 0, id1 = 0;
    int idq[8];
    auto load_ids = [&]() {
        id0 = a.map[row0 + min(lane, rows_b - 1)];
        id1 = a.map[row0 + min(lane + kWave, rows_b - 1)];
#pragma unroll
        for (int q = 0; q < 8; ++q) idq[q] = a.map[row0 + min(lrow + 16 * q, rows_b - 1)];
    };
    if constexpr (NTW == 1) load_ids();

    // ---- steady state.  Per iteration the wave issues NB B-loads, then 4 W-loads, always in this order,
    // so the age of every outstanding load is known:
    //   W(u+1) was issued PU iterations ago as the last 4 loads      -> (PU-1)*(NB+4) + NB younger loads
    //   B(u)   was issued last iteration as the first NB loads       -> 4 + NB + 4 younger loads
    constexpr int kWaitA = (PU - 1) * (NB + 4) + NB;
    constexpr int kWaitB = 8 + NB;
    static_assert(kWaitA <= 63, "vmcnt range");
    auto iteration = [&](int u, auto par_tag, auto slot_tag) {
        constexpr int PAR = decltype(par_tag)::value;      // u & 1
        constexpr int SLOT = decltype(slot_tag)::value;    // (u + 1) % PU: register slot of unit u + 1
        unsigned char *cur = smem + PAR * kUbufBytes;
        unsigned char *nxt = smem + (PAR ^ 1) * kUbufBytes;
        load_b(u + 1, breg[PAR ^ 1]);
        wait_regs<kWaitA, 4>(areg[SLOT]);
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(nxt + 4 * j * kStagePitch + wr_off) = areg[SLOT][j];
        load_unit(u + 1 + PU, areg[SLOT]);
        if constexpr (NB == 4) wait_regs<kWaitB, 4>(breg[PAR]);
        else wait_regs<kWaitB, 8>(breg[PAR]);
        if (rotate && u > 0) {
            const int ua = unit_of(u);
            __builtin_amdgcn_sched_barrier(0);
            if (ua == 0 || ua == rb1 || ua == rb2 || ua == rb3) close_range();
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) {
                const u32x4 av = *reinterpret_cast<const u32x4 *>(cur + 16 * mt * kStagePitch + rd_off + ks * 64);
#pragma unroll
                for (int t = 0; t < NTW; ++t)
                    acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, breg[PAR][ks * NTW + t]),
                        acc[mt][t], 0, 0, 0);
            }
        }
        __syncthreads();   // unit u consumed by everyone, unit u + 1 staged by everyone
    };
    // the register slot of unit u + 1 cycles with period PU and the buffer parity with period 2:
    // unroll over lcm(2, PU) = 6 iterations
    static_assert(PU == 3, "the unrolled schedule below assumes three units in flight");
    int u = 0;
    for (; u + 6 <= nunits; u += 6) {
        iteration(u + 0, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{});
        iteration(u + 1, std::integral_constant<int, 1>{}, std::integral_constant<int, 2>{});
        iteration(u + 2, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        iteration(u + 3, std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{});
        iteration(u + 4, std::integral_constant<int, 0>{}, std::integral_constant<int, 2>{});
        iteration(u + 5, std::integral_constant<int, 1>{}, std::integral_constant<int, 0>{});
    }
    do {      // the remaining 0..5 units: one exit, so that no path skips an iteration and runs a later one
        if (u + 0 >= nunits) break;
        iteration(u + 0, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{});
        if (u + 1 >= nunits) break;
        iteration(u + 1, std::integral_constant<int, 1>{}, std::integral_constant<int, 2>{});
        if (u + 2 >= nunits) break;
        iteration(u + 2, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        if (u + 3 >= nunits) break;
        iteration(u + 3, std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{});
        if (u + 4 >= nunits) break;
        iteration(u + 4, std::integral_constant<int, 0>{}, std::integral_constant<int, 2>{});
    } while (false);
    if constexpr (NTW != 1) load_ids();
    // loads past the end are still in flight: let them land before their registers die
#pragma unroll
    for (int x = 0; x < PU; ++x) wait_regs<0, 4>(areg[x]);
    if constexpr (NB == 4) {
        wait_regs<0, 4>(breg[0]);
        wait_regs<0, 4>(breg[1]);
    } else {
        wait_regs<0, 8>(breg[0]);
        wait_regs<0, 8>(breg[1]);
    }

    if constexpr (NTW == 1) {
        if (rotate) {
            close_range();
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) acc[mt][0] = pair0[mt] + pair1[mt];
        }
    }

    // ---- logits -> LDS tile zt[i][t] (the last barrier above freed the unit buffers)
    const int tp = kMfmaTileRows + 1;
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
        const int i = 16 * (NTW * w + t) + lrow;
        if (i < a.n) {
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) {
                float *dst = zt + (size_t)i * tp + 16 * mt + 4 * lgrp;
                dst[0] = acc[mt][t].x;
                dst[1] = acc[mt][t].y;
                dst[2] = acc[mt][t].z;
                dst[3] = acc[mt][t].w;
            }
        }
    }
    __syncthreads();

    if (a.zbuf != nullptr) {
        // store-only tail: the tile's logits go to z [n, k]; a workgroup per hidden row finishes the step
        // (row_select_kernel).  One wave copies a hidden row's 128 logits (512 contiguous bytes) at a time.
        for (int i = w; i < a.n; i += kStepWaves) {
            const float *src = zt + (size_t)i * tp;
            float *dst = a.zbuf + (size_t)i * a.k + row0;
            if (lane < rows_b) dst[lane] = src[lane];
            if (lane + kWave < rows_b) dst[lane + kWave] = src[lane + kWave];
        }
        return;
    }

    if (a.L <= 16) {
        // candidate keys of the threshold selection: 4 rows x 16 keys per wave, behind the logit tile
        unsigned long long *cand4 =
            reinterpret_cast<unsigned long long *>(smem + (((size_t)a.n * tp * sizeof(float) + 15) & ~(size_t)15)) +
            (size_t)w * 4 * 16;
        for (int i0 = 4 * w; i0 < a.n; i0 += 4 * kStepWaves)
            block_epilogue_rows4<8, true>(zt, tp, i0, a.n, rows_b, a.L, idq, a.out_logp_full, (size_t)a.k, row0, a.pms,
                                    a.pkeys, a.nlists, (int)blockIdx.x, lane, cand4);
    } else {
        for (int i = w; i < a.n; i += kStepWaves) {
            const float *zrow = zt + (size_t)i * tp;
            float *full = a.out_logp_full ? a.out_logp_full + (size_t)i * a.k + row0 : nullptr;
            unsigned long long *pms_slot = a.pms + (size_t)i * a.nlists + blockIdx.x;
            unsigned long long *pk_slot = a.pkeys + ((size_t)i * a.nlists + blockIdx.x) * a.L;
            block_epilogue_small(zrow, 1, 0, rows_b, a.L, id0, id1, full, pms_slot, pk_slot, lane);
        }
    }
}

// The merge of one hidden row per workgroup with a tree level behind it: wave 0 merges the row (its results are
// written through to memory) and takes a ticket; the workgroup that draws the last ticket ranks all n * m
// candidates, reading the other rows' results with loads that bypass its caches.
// T threads: 64 when n * m <= 64, else 512 (the waves beyond the first only help with the ranking; with more
// threads the merging wave would not have the registers it needs).
template <int T>
__global__ void __launch_bounds__(T) step_finalize_tree_kernel(const FinalizeArgs f) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_last;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int i = blockIdx.x;
    if (w == 0) {
        unsigned long long *stage = reinterpret_cast<unsigned long long *>(smem);
        finalize_row<true>(f.pms + (size_t)i * f.nlists, f.pkeys + (size_t)i * f.nlists * f.L, f.nlists, f.L, f.m, stage,
                           f.out_ids + (size_t)i * f.m, f.out_logp + (size_t)i * f.m, f.out_lse ? f.out_lse + i : nullptr,
                           f.lse_buf + i, lane);
        wait_stores_done();       // the row's results are written through: visible to whoever draws the last ticket
        if (lane == 0) {
            const unsigned v = __hip_atomic_fetch_add(f.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int last = v == (unsigned)(f.n - 1);
            if (last) __hip_atomic_store(f.ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = last;
        }
    }
    __syncthreads();
    if (!s_last) return;
    TreeArgs t;
    t.parent_cum = f.tree_cum;
    t.vals = f.out_logp;
    t.ids = f.out_ids;
    t.N = f.n * f.m;
    t.m = f.m;
    t.K = f.tree_K;
    t.index_order = 0;
    t.out_a = f.tree_parent;
    t.out_token = f.tree_token;
    t.out_score = f.tree_score;
    int N2 = kWave;
    while (N2 < t.N) N2 <<= 1;
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(smem);
    unsigned *cnt = reinterpret_cast<unsigned *>(smem + (size_t)N2 * 8);
    int *wave_tot = reinterpret_cast<int *>(smem + (size_t)N2 * 12);
    tree_select_by_count<T, true>(t, N2, keys, cnt, wave_tot);
}

// Merges the per-tile partials: one wave per hidden row.
__global__ void __launch_bounds__(kStepWaves *kWave) step_finalize_kernel(const FinalizeArgs f) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (w >= f.conc) return;
    const int i = blockIdx.x * f.conc + w;
    if (i >= f.n) return;
    unsigned long long *stage = reinterpret_cast<unsigned long long *>(smem) + (size_t)w * f.stage_keys;
    const int o = f.indexed ? (int)((f.row_pack >> (8 * (i & 7))) & 0xFFull) : i;      // output row
    finalize_row<true>(f.pms + (size_t)i * f.nlists, f.pkeys + (size_t)i * f.nlists * f.L, f.nlists, f.L, f.m, stage,
                 f.out_ids + (size_t)o * f.m, f.out_logp + (size_t)o * f.m, f.out_lse ? f.out_lse + o : nullptr,
                 f.lse_buf + i, lane);
}

hipError_t launch_pack_h_impl(const MfmaArgs &a, int groups, hipStream_t st) {
    const long long pieces = (long long)(a.d / 128) * 4 * groups * 64;
    const unsigned blocks = (unsigned)((pieces + 255) / 256);
    hipLaunchKernelGGL(pack_h_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const u32x4 *>(a.h),
                       static_cast<u32x4 *>(a.hpack), a.n, a.d, groups, pieces);
    return hipGetLastError();
}

template <int NTW>
hipError_t launch_mfma_wide_inst(const MfmaArgs &a, size_t lds, hipStream_t st) {
    auto kern = head_mfma_wide_kernel<NTW>;
    static LdsLimitOnce lds_limit;
    hipError_t e = allow_dynamic_lds(lds_limit, {reinterpret_cast<const void *>(kern)}, kMaxDynamicLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(a.nlists), dim3(kStepWaves * kWave), lds, st, a);
    return hipGetLastError();
}

template <int NT, int MAXW, bool XG = false, int XC = 0>
hipError_t launch_mfma_inst(const MfmaArgs &a, size_t lds, hipStream_t st) {
    auto kern = head_mfma_kernel<NT, MAXW, XG, XC, false>;
    static LdsLimitOnce lds_limit;
    hipError_t e = allow_dynamic_lds(lds_limit, {reinterpret_cast<const void *>(kern)}, kMaxDynamicLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(a.nlists), dim3((MAXW == kStepWaves ? kStepWaves : a.nwaves) * kWave), lds, st, a,
                       SingleHead{});
    return hipGetLastError();
}
template <int MAXW>
hipError_t launch_mfma_multi_inst(const MfmaArgs &a, const MultiHeadTable &t, size_t lds, hipStream_t st) {
    auto kern = head_mfma_kernel<1, MAXW, false, 0, true>;
    static LdsLimitOnce lds_limit;
    hipError_t e = allow_dynamic_lds(lds_limit, {reinterpret_cast<const void *>(kern)}, kMaxDynamicLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(a.nlists), dim3((MAXW == kStepWaves ? kStepWaves : a.nwaves) * kWave), lds, st, a, t);
    return hipGetLastError();
}

}  // namespace

size_t mfma_stage_bytes(int nwaves) { return (size_t)nwaves * 2 * kStageUnitBytes; }
size_t mfma_wide_lds_bytes() { return 2 * (size_t)kMfmaTileRows * kStagePitch; }

hipError_t launch_head_mfma(int NT, const MfmaArgs &a, size_t lds, hipStream_t st) {
    // the kernels for up to 64 hidden rows run a chunk that has a successor in whole rounds of units
    if (NT <= 4 && (a.KC <= 0 || a.KC % kUnitCols != 0 ||
                    (a.KC < a.d && (a.KC / kUnitCols) % kPrefetchUnits != 0)))
        return hipErrorInvalidValue;
    // the column split needs one chunk, up to 8 hidden rows, whole units per wave and the fused epilogue
    if (a.ksplit != 1 &&
        ((a.ksplit != 2 && a.ksplit != 4) || NT != 1 || a.n > 8 || a.KC < a.d || (a.d / kUnitCols) % a.ksplit != 0 ||
         a.zbuf != nullptr))
        return hipErrorInvalidValue;
    // waves per workgroup: eight, or (one group of hidden rows, all of h in LDS, up to 8 hidden rows) a multiple of
    // the column split up to kMfmaMaxWaves
    // ... or (two or four groups of hidden rows, no column split) five to seven: tiles of 80 .. 112 rows
    const bool few = a.nwaves != kStepWaves && NT > 1;
    if (few && ((NT != 2 && NT != 4) || a.nwaves < 5 || a.nwaves > kMfmaFewWaves || a.ksplit != 1 || a.extra_rows != 0 ||
                (a.zbuf == nullptr && a.L > 16) ||
                (size_t)16 * NT * min(a.KC, a.d) * 2 > (size_t)kMaxPieces * a.nwaves * kWave * 16))
        return hipErrorInvalidValue;
    if (a.nwaves != kStepWaves && !few &&
        (NT != 1 || a.n > 8 || a.KC < a.d || a.nwaves < a.ksplit || a.nwaves > kMfmaMaxWaves ||
         a.nwaves % a.ksplit != 0 || (size_t)a.d * 16 > (size_t)kMaxPieces * a.nwaves * kWave * 16))
        return hipErrorInvalidValue;
    // rows past the 128th as one more group: shared by the eight waves (up to 8 hidden rows: eight column parts of
    // whole units, all of h in LDS), multiplied from LDS beside h's chunk (two groups of hidden rows) or after the
    // march (four groups); rows of at least 8 units
    const bool xmany = a.extra_rows != 0 && a.n > 8;      // extra rows with more than 8 hidden rows
    if (a.extra_rows != 0 && !xmany &&
        (a.extra_rows < 1 || a.extra_rows > 16 || NT != 1 || a.KC < a.d || a.ksplit != 1 ||
         a.nwaves != kStepWaves || (a.d / kUnitCols) % 8 != 0))
        return hipErrorInvalidValue;
    if (xmany &&
        (a.extra_rows < 1 || a.extra_rows > 16 || (NT != 2 && NT != 4) || a.ksplit != 1 || a.nwaves != kStepWaves ||
         a.d / kUnitCols < 8 || (a.zbuf == nullptr && a.L > 16)))
        return hipErrorInvalidValue;
    const size_t xtile = ((size_t)a.n * (kMfmaTileRows + 17) * sizeof(float) + 15) / 16 * 16 +
                         kStepWaves * 4 * 16 * sizeof(unsigned long long);      // logit tile and candidate keys of the epilogue
    if (xmany && NT == 2) {
        // the chunk and the extra rows' pieces fit the register prefetch; the accumulators' LDS lies behind the chunk,
        // inside the launch's LDS and clear of the logit tile
        const int ppr = min(a.KC, a.d) >> 3;
        const int qx = (16 * NT * ppr + kStepWaves * kWave - 1) / (kStepWaves * kWave);
        const int xpieces = (16 * ppr + kStepWaves * kWave - 1) / (kStepWaves * kWave);
        if (qx + xpieces > kMaxPieces || (a.xoff & 15) != 0 ||
            (size_t)a.xoff < (size_t)kStageBytes + (size_t)(16 * NT + 16) * a.hpitch ||
            (size_t)a.xoff + (size_t)3 * NT * kWave * sizeof(f32x4) > lds || xtile > (size_t)a.xoff)
            return hipErrorInvalidValue;
    }
    // (four groups: the pass after the march leaves its four range sums per logit behind the tile)
    if (xmany && NT == 4 && xtile + (size_t)4 * a.n * 16 * sizeof(float) > lds) return hipErrorInvalidValue;
    {
        const int tile_rows = 16 * (a.nwaves / a.ksplit) + a.extra_rows;
        if (a.nlists != (a.k + tile_rows - 1) / tile_rows) return hipErrorInvalidValue;
    }
    if ((size_t)a.d * 2 >= ((size_t)1 << 24)) return hipErrorInvalidValue;      // row offsets inside a tile: 24-bit factors
    switch (NT) {
        case 1:
            if (xmany) return hipErrorInvalidValue;      // planned with two groups of hidden rows
            if (a.extra_rows != 0) return launch_mfma_inst<1, kStepWaves, true>(a, lds, st);
            return a.nwaves == kStepWaves ? launch_mfma_inst<1, kStepWaves>(a, lds, st)
                                          : launch_mfma_inst<1, kMfmaMaxWaves>(a, lds, st);
        case 2:
            if (few) return launch_mfma_inst<2, kMfmaFewWaves>(a, lds, st);
            return xmany ? launch_mfma_inst<2, kStepWaves, false, 1>(a, lds, st)
                             : launch_mfma_inst<2, kStepWaves>(a, lds, st);
        case 4:
            if (few) return launch_mfma_inst<4, kMfmaFewWaves>(a, lds, st);
            return xmany ? launch_mfma_inst<4, kStepWaves, false, 2>(a, lds, st)
                             : launch_mfma_inst<4, kStepWaves>(a, lds, st);
        case 8:
        case 16: {
            if (a.hpack == nullptr) return hipErrorInvalidValue;
            const hipError_t e = launch_pack_h_impl(a, NT, st);
            if (e != hipSuccess) return e;
            return NT == 8 ? launch_mfma_wide_inst<1>(a, lds, st) : launch_mfma_wide_inst<2>(a, lds, st);
        }
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_head_mfma_multi(const MfmaArgs &a, const MultiHeadTable &t, size_t lds, hipStream_t st) {
    // up to 8 hidden rows in place, all of h in LDS, plain tiles (a column split only with eight waves), the kernel's
    // own epilogue; every head cut into tiles of the launch's height on its own
    if (a.n < 1 || a.n > 8 || a.KC != a.d || a.indexed != 0 || a.zbuf != nullptr || a.out_logp_full != nullptr ||
        a.extra_rows != 0 || a.ticket_clear != nullptr || a.d % kUnitCols != 0 || a.L < 1 || a.L > 16 ||
        a.nwaves < kStepWaves || a.nwaves > kMfmaMaxWaves || (a.ksplit != 1 && (a.nwaves != kStepWaves || (a.ksplit != 2 && a.ksplit != 4))) ||
        (a.d / kUnitCols) % a.ksplit != 0 || (size_t)a.d * 16 > (size_t)kMaxPieces * a.nwaves * kWave * 16 ||
        (size_t)a.d * 2 >= ((size_t)1 << 24) || t.n_heads < 1 || t.n_heads > 16 || t.tile_first[0] != 0)
        return hipErrorInvalidValue;
    const int tile_rows = 16 * (a.nwaves / a.ksplit);
    for (int q = 0; q < t.n_heads; ++q) {
        if (t.W[q] == nullptr || t.map[q] == nullptr || t.k[q] < 1 ||
            t.tile_first[q + 1] - t.tile_first[q] != (t.k[q] + tile_rows - 1) / tile_rows)
            return hipErrorInvalidValue;
    }
    for (int i = 0; i < a.n; ++i)
        if ((int)((t.head_of_row >> (8 * i)) & 0xFFull) >= t.n_heads) return hipErrorInvalidValue;
    if (a.nlists != t.tile_first[t.n_heads] || a.nlists > kStepMaxBlocks) return hipErrorInvalidValue;
    return a.nwaves == kStepWaves ? launch_mfma_multi_inst<kStepWaves>(a, t, lds, st)
                                  : launch_mfma_multi_inst<kMfmaMaxWaves>(a, t, lds, st);
}

hipError_t launch_step_finalize(const FinalizeArgs &f, size_t lds, hipStream_t st) {
    static LdsLimitOnce lds_limit;
    hipError_t e = allow_dynamic_lds(lds_limit, {reinterpret_cast<const void *>(step_finalize_kernel)}, kMaxDynamicLds);
    if (e != hipSuccess) return e;
    if (f.tree_cum != nullptr) {
        // one hidden row per workgroup; LDS: the merge's staging, then the ranking's keys and counters
        const int N = f.n * f.m;
        if (f.conc != 1 || f.indexed || N > kFinalizeTreeMaxN || f.ticket == nullptr) return hipErrorInvalidValue;
        int N2 = kWave;
        while (N2 < N) N2 <<= 1;
        const size_t need = (size_t)N2 * 12 + 256;
        const size_t bytes = lds > need ? lds : need;
        static LdsLimitOnce tree_lds_limit;
        e = allow_dynamic_lds(tree_lds_limit, {reinterpret_cast<const void *>(step_finalize_tree_kernel<64>),
                                               reinterpret_cast<const void *>(step_finalize_tree_kernel<512>)},
                              kMaxDynamicLds);
        if (e != hipSuccess) return e;
        if (N <= kWave)
            hipLaunchKernelGGL(step_finalize_tree_kernel<64>, dim3(f.n), dim3(64), bytes, st, f);
        else
            hipLaunchKernelGGL(step_finalize_tree_kernel<512>, dim3(f.n), dim3(512), bytes, st, f);
        return hipGetLastError();
    }
    const int grid = (f.n + f.conc - 1) / f.conc;
    hipLaunchKernelGGL(step_finalize_kernel, dim3(grid), dim3(f.conc * kWave), lds, st, f);
    return hipGetLastError();
}

}  // namespace vt
