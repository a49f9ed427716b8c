/*
 * vocabtrim.h -- C ABI of libvocabtrim.so: the trimmed-LM-head hot path of
 * VocabTrim (training-free vocabulary trimming of a speculative-decoding
 * drafter's LM head) for AMD MI355X (gfx950).
 *
 * Three operations, named after the paper's problem statement:
 *
 *   vt_count_tokens        Algorithm 1 (Count Token Frequencies)
 *   vt_build_trimmed_head  Eq. 1 (V_trim = V[Top-K(c,k)], W_trim = W[Top-K(c,k), :])
 *                          and the token index mapper T_{d->t} of Algorithm 2
 *   vt_draft_head_step     Algorithm 2, the two drafting lines: the trimmed
 *                          drafter's output z_hat over the trimmed vocabulary
 *                          and y_hat = T_{d->t}(z_hat), with the EAGLE-2 style
 *                          draft-token selection named in the experimental
 *                          settings (top-m tokens per node with log-probs;
 *                          greedy top-1 for chain drafting)
 *
 * General conventions
 * -------------------
 * - Every data pointer is DEVICE memory owned by the caller (for example a
 *   torch tensor's data_ptr()).  The library never allocates, frees, or keeps
 *   a pointer after the call returns.  No call synchronises the device or
 *   reads device memory on the host.
 * - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   All work is enqueued on it; outputs are valid once the stream has reached
 *   that point.
 * - `ws` is caller-provided device scratch of at least the size returned by
 *   the matching *_ws_bytes() function (a pure host function), 256-byte
 *   aligned.  A workspace may be reused by successive calls on one stream;
 *   two calls that may overlap in time need separate workspaces.
 * - Host-detectable errors return a non-zero vt_status and enqueue nothing.
 *   Data-dependent conditions (token ids outside [0,V)) cannot be reported
 *   synchronously; see vt_count_tokens.
 * - Layouts are row-major and contiguous.  Vocabulary ids and the map are
 *   int32 (V < 2^31); counters are int64; log-probs are fp32.
 * - Supported element types of (h, W): both VT_BF16 or both VT_F32.  bf16
 *   products are accumulated in fp32.
 */
#ifndef VOCABTRIM_H_
#define VOCABTRIM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VT_OK = 0,
    VT_ERR_NULL = 1,      /* a required pointer is NULL */
    VT_ERR_SHAPE = 2,     /* a size is out of range (V, d, n <= 0; k not in [1,V]; m not in [1,min(k,VT_MAX_TOP_M)]) */
    VT_ERR_DTYPE = 3,     /* unknown or unsupported element / index type, or h and W differ */
    VT_ERR_ALIGN = 4,     /* a pointer is not 16-byte aligned, or d is not a multiple of 16 bytes of elements */
    VT_ERR_WORKSPACE = 5, /* ws is NULL, misaligned or smaller than *_ws_bytes() */
    VT_ERR_DEVICE = 6     /* a HIP call failed (launch error, no device) */
} vt_status;

typedef enum { VT_F32 = 0, VT_BF16 = 1 } vt_dtype;
typedef enum { VT_I32 = 0, VT_I64 = 1 } vt_itype;

/* Largest m (tokens kept per hidden row) vt_draft_head_step accepts. */
#define VT_MAX_TOP_M 64

/* Human-readable name of a status code (static storage). */
const char *vt_status_string(int status);

/* Text of the HIP error behind the calling thread's most recent VT_ERR_DEVICE
 * (static storage; "no error" if there was none). */
const char *vt_last_device_error(void);

/* ------------------------------------------------------------------------
 * Algorithm 1 -- Count Token Frequencies.
 *
 * For every token id t in ids[0..n_ids): counts[t] += 1.  `counts` is
 * accumulated into, so a calibration corpus can be fed in chunks and the
 * vector saved / resumed by the caller; zero it before the first chunk (the
 * algorithm's "initialize with zeros").  Tokenisation is the caller's: the
 * function consumes ids.
 *
 *   ids        [n_ids] int32 or int64 (id_type), device; may be NULL iff n_ids == 0
 *   n_ids      number of ids, >= 0 (0 is a valid no-op)
 *   V          vocabulary size, > 0
 *   counts     [V] int64, device, in/out
 *   n_invalid  device uint64, in/out, nullable: ids < 0 or >= V are skipped
 *              and added here, so sum(counts) + *n_invalid grows by n_ids
 *   ws         >= vt_count_tokens_ws_bytes(V, n_ids) bytes; contents need no
 *              initialisation
 * ---------------------------------------------------------------------- */
int vt_count_tokens(const void *ids, int id_type, int64_t n_ids, int32_t V, int64_t *counts,
                    uint64_t *n_invalid, void *ws, size_t ws_bytes, void *stream);
size_t vt_count_tokens_ws_bytes(int32_t V, int64_t n_ids);

/* ------------------------------------------------------------------------
 * Eq. 1 -- vocabulary trimming.
 *
 * Top-K(c,k): the k ids with the largest counts; among equal counts the
 * lower id is taken first (ids never seen have count 0 and fill the tail by
 * ascending id).  The selected ids are written in ASCENDING id order:
 *
 *   map[j]        the j-th smallest selected id  (token index mapper T_{d->t})
 *   W_trim[j, :]  = W[map[j], :]                 (bit copy of the stored type)
 *
 * so k == V gives map = identity and W_trim == W.
 *
 *   counts  [V] int64, device (values >= 0)
 *   W       [V, d] row-major, w_type, device
 *   d       hidden size; d * sizeof(element) must be a multiple of 16
 *   k       trimmed vocabulary size, 1 <= k <= V
 *   map     [k] int32, device, out
 *   W_trim  [k, d] row-major, w_type, device, out; must not overlap W
 *   ws      >= vt_build_trimmed_head_ws_bytes(V, d, k) bytes; no initialisation
 * W may be NULL together with W_trim to compute the map only.
 * ---------------------------------------------------------------------- */
int vt_build_trimmed_head(const int64_t *counts, int32_t V, const void *W, int w_type, int32_t d,
                          int32_t k, int32_t *map, void *W_trim, void *ws, size_t ws_bytes,
                          void *stream);
size_t vt_build_trimmed_head_ws_bytes(int32_t V, int32_t d, int32_t k);

/* ------------------------------------------------------------------------
 * The same build with the rows in FREQUENCY-RANK order: map (and W_trim's
 * rows) sorted by (count descending, id ascending), the order in which
 * Top-K(c, k) takes ids.  Every prefix of the result is the trimmed head for
 * a smaller k, so one build at the largest k of interest serves a whole
 * ablation over k by pointer arithmetic; the draft step breaks ties of equal
 * logits by target id, so it accepts either order.  Arguments, errors and
 * workspace size as for vt_build_trimmed_head.
 * ---------------------------------------------------------------------- */
int vt_build_trimmed_head_by_rank(const int64_t *counts, int32_t V, const void *W, int w_type, int32_t d,
                                  int32_t k, int32_t *map, void *W_trim, void *ws, size_t ws_bytes,
                                  void *stream);

/* ------------------------------------------------------------------------
 * Choosing k from the counts instead of fixing it (the method section notes
 * that Top-P over the counts or a minimum-frequency threshold can replace a
 * fixed k):
 *
 *   VT_K_TOP_P      smallest k >= 1 whose k most frequent ids carry at least
 *                   p of all counted tokens: S_k >= ceil(p * S_V), S_k = sum of
 *                   the k largest counts, p * S_V one fp64 product; 0 <= p <= 1
 *   VT_K_MIN_COUNT  k = number of ids with count >= min_count (may be 0)
 *
 *   counts  [V] int64, device (values >= 0, their sum below 2^63)
 *   out     [3] int64, device, out: k, S_k (tokens covered), S_V (all tokens);
 *           S_k / S_V is the coverage of the calibration set.  The caller reads
 *           k back (one small copy) before sizing W_trim for the build.
 *   ws      >= vt_choose_k_ws_bytes(V) bytes; no initialisation
 * ---------------------------------------------------------------------- */
typedef enum { VT_K_TOP_P = 0, VT_K_MIN_COUNT = 1 } vt_kmode;
int vt_choose_k(const int64_t *counts, int32_t V, int mode, double p, int64_t min_count, int64_t *out,
                void *ws, size_t ws_bytes, void *stream);
size_t vt_choose_k_ws_bytes(int32_t V);

/* ------------------------------------------------------------------------
 * Algorithm 2, drafting lines -- one draft step of the trimmed LM head.
 *
 *   z[i, j]   = sum_t h[i, t] * W_trim[j, t]            (never stored unless asked)
 *   lse[i]    = log sum_j exp z[i, j]   over the k trimmed logits only
 *   per row i: the m largest z[i, .], descending; equal logits -> lower target
 *              id first
 *   out_ids[i, r]  = map[j_r]                            (y_hat = T_{d->t}(z_hat))
 *   out_logp[i, r] = z[i, j_r] - lse[i]
 *
 *   h              [n, d] row-major, h_type, device
 *   n              hidden rows this step (chain drafting: 1; tree drafting: nodes), 1 <= n
 *                  (one launch covers n <= 8, and n <= 256 for bf16 with d a multiple of
 *                  128; other shapes run as consecutive groups of rows, each streaming
 *                  W_trim again)
 *   W_trim         [k, d] row-major, w_type (== h_type), device
 *   map            [k] int32 target ids, device
 *   m              tokens kept per row, 1 <= m <= min(k, VT_MAX_TOP_M)
 *   out_ids        [n, m] int32, device, out
 *   out_logp       [n, m] fp32, device, out
 *   out_lse        [n] fp32, device, out, nullable
 *   out_logp_full  [n, k] fp32, device, out, nullable: log-softmax of every
 *                  trimmed logit (costs an extra pass; meant for checks)
 *   ws             >= vt_draft_head_step_ws_bytes(n, k, d, m) bytes.  Its contents
 *                  need no initialisation, before the first step or between
 *                  steps, whatever their shapes (as long as the size suffices)
 *                  and whatever an earlier step that never completed left behind.
 * ---------------------------------------------------------------------- */
int vt_draft_head_step(const void *h, int h_type, int32_t n, const void *W_trim, int w_type,
                       int32_t k, int32_t d, const int32_t *map, int32_t m, int32_t *out_ids,
                       float *out_logp, float *out_lse, float *out_logp_full, void *ws,
                       size_t ws_bytes, void *stream);
size_t vt_draft_head_step_ws_bytes(int32_t n, int32_t k, int32_t d, int32_t m);

/* Which kernels vt_draft_head_step launches for a shape, and how the head is cut
 * into workgroups (a pure host function, for logs and benchmarks: the choice
 * is the library's and may change between versions).  Writes a
 * NUL-terminated line of at most text_bytes bytes to the HOST buffer `text`,
 * for example "head_mfma_kernel<1,12> workgroups=229 tile_rows=144 waves=9
 * column_split=1 + step_finalize_kernel".  Errors as for the step's shape checks. */
int vt_draft_head_step_plan(int32_t n, int32_t k, int32_t d, int32_t m, int w_type, char *text, size_t text_bytes);

/* ------------------------------------------------------------------------
 * vt_draft_head_step_static -- the same draft step for callers that cannot
 * allocate device memory or hand in a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments,
 * results (bit for bit) and errors as for vt_draft_head_step, without ws /
 * ws_bytes: the partial results of the step live in an array of
 * VT_STATIC_WS_BYTES bytes that the library itself holds on every GPU it runs
 * on, from the first use of the library on that GPU until the process ends.
 * The call allocates and frees nothing (its first call on a device asks the
 * runtime for the array's address; make that call outside stream capture).
 *   - A shape whose vt_draft_head_step_ws_bytes(n, k, d, m) exceeds
 *     VT_STATIC_WS_BYTES returns VT_ERR_WORKSPACE and enqueues nothing (for
 *     example n = 256 rows with 16 tokens per row at k = 32768, whose per-row
 *     tail stores 32 MiB of logits); the paper's shapes (up to 64 tree nodes x
 *     top-8 at k = 32768) need at most 1.2 MiB.
 *   - All calls on one GPU share that GPU's array: calls that may overlap in
 *     time (different streams, different host threads) race; order them on one
 *     stream or use vt_draft_head_step with workspaces of your own.
 * ---------------------------------------------------------------------- */
#define VT_STATIC_WS_BYTES (4u << 20)
int vt_draft_head_step_static(const void *h, int h_type, int32_t n, const void *W_trim, int w_type,
                              int32_t k, int32_t d, const int32_t *map, int32_t m, int32_t *out_ids,
                              float *out_logp, float *out_lse, float *out_logp_full, void *stream);

/* ------------------------------------------------------------------------
 * Several trimmed heads at once (Sec. 4.1, task-specific vocabularies: a small
 * function-calling vocabulary beside the general one; the conclusion's note on
 * swappable per-task heads).  A head is a (map, W_trim, k) triple; all heads
 * come from one W and share d.
 *
 * vt_build_trimmed_heads -- Eq. 1 for n_heads count vectors:
 *     counts   [n_heads, V] int64, device: one row of counters per head
 *     k        [n_heads] int32, HOST: trimmed size of every head, 1 <= k[i] <= V
 *     map      [n_heads] HOST array of device pointers, map[i] -> [k[i]] int32, out
 *     W_trim   [n_heads] HOST array of device pointers, W_trim[i] -> [k[i], d], out;
 *              NULL together with W to compute the maps only
 *     ws       >= vt_build_trimmed_head_ws_bytes(V, d, max k) bytes
 *   Every head is checked before the first is built; results as for
 *   vt_build_trimmed_head head by head (ascending id order).
 *
 * vt_draft_head_step_multi -- one draft step in which hidden row i uses head
 *   head_of_row[i]: out_ids[i, :], out_logp[i, :], out_lse[i] are what
 *   vt_draft_head_step returns for row i on that head -- the same tokens, and
 *   log-probs that differ at most by the rounding of the log-sum-exp (a few
 *   1e-7), whose partial sums follow the tiles the head is cut into.  Every
 *   head that has rows streams its W_trim once, whatever the order of the
 *   rows.  Up to 8 rows (bf16, d a multiple of 128 up to 4096, m <= 11) on two
 *   or more heads run as ONE launch over all those heads' tiles, so the fixed
 *   costs of a step are paid once, not per head; otherwise the heads run one
 *   after another (rows of a head that are not consecutive in h are picked
 *   out by the kernel or staged through the workspace).
 *     h            [n, d] device;  1 <= n <= VT_MULTI_MAX_ROWS
 *     W_trim, map  [n_heads] HOST arrays of device pointers (entries of heads
 *                  without rows are not read)
 *     k            [n_heads] int32, HOST
 *     head_of_row  [n] int32, HOST, values in [0, n_heads)
 *     m            1 <= m <= min(VT_MAX_TOP_M, k of every head that has rows)
 *     out_lse      nullable
 *     ws           >= vt_draft_head_step_multi_ws_bytes(n, d, k, n_heads, m) bytes
 *                  (0 = arguments out of range); no initialisation
 *   Only kernels are enqueued (no copies): the call may be captured in a graph.
 * ---------------------------------------------------------------------- */
#define VT_MAX_HEADS 16
#define VT_MULTI_MAX_ROWS 256
int vt_build_trimmed_heads(const int64_t *counts, int32_t V, int32_t n_heads, const void *W, int w_type,
                           int32_t d, const int32_t *k, int32_t *const *map, void *const *W_trim, void *ws,
                           size_t ws_bytes, void *stream);
int vt_draft_head_step_multi(const void *h, int h_type, int32_t n, int32_t d, const void *const *W_trim,
                             int w_type, const int32_t *k, const int32_t *const *map, int32_t n_heads,
                             const int32_t *head_of_row, int32_t m, int32_t *out_ids, float *out_logp,
                             float *out_lse, void *ws, size_t ws_bytes, void *stream);
size_t vt_draft_head_step_multi_ws_bytes(int32_t n, int32_t d, const int32_t *k, int32_t n_heads, int32_t m);
/* Pure host function: how vt_draft_head_step_multi would run these rows, as text
 * ("head_mfma_kernel<1,12> heads=2 workgroups=237 tile_rows=160 ..." for one
 * launch over several heads' tiles, "head by head (N)" otherwise).  k and
 * head_of_row are HOST arrays as above.  Returns VT_OK or an argument error. */
int vt_draft_head_step_multi_plan(int32_t n, int32_t d, const int32_t *k, int32_t n_heads, const int32_t *head_of_row,
                                  int32_t m, int w_type, char *text, size_t text_bytes);

/* Not needed any more (a draft-step workspace needs no initialisation); kept for
 * callers written against earlier versions.  Zeroes the first 2 KiB of the
 * workspace with a small fill kernel on `stream`. */
int vt_draft_head_step_ws_init(void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------
 * Draft-tree growth on top of the draft step (experimental settings, "Draft
 * Tree": EAGLE-2 style tree of depth 3 with top-K = 8 per level and at most
 * 32 draft tokens; the depth ablation keeps 60).  Selection arithmetic only;
 * verification against a target model is the caller's.
 *
 * vt_tree_expand -- one level: candidate (i, j) = token step_ids[i, j] under
 *   frontier node i scores parent_cum[i] + step_logp[i, j] (ONE fp32 addition);
 *   the K best candidates, best first, are the next frontier.  Equal scores
 *   (-0.0 == +0.0) go to the lower flat index i * m + j.
 *     parent_cum  [n] fp32, device: cumulative log-prob of the frontier nodes
 *     step_logp   [n, m] fp32, device  (vt_draft_head_step's out_logp)
 *     step_ids    [n, m] int32, device (vt_draft_head_step's out_ids)
 *     n, m        1 <= n, 1 <= m, n * m <= VT_TREE_MAX_CANDIDATES
 *     K           1 <= K <= n * m
 *     out_parent  [K] int32, device, out: frontier index i of each survivor
 *     out_token   [K] int32, device, out: its token id
 *     out_cum     [K] fp32, device, out: its cumulative log-prob (a sum of -0.0 is
 *                 returned as +0.0)
 *
 * vt_tree_rerank -- the T best of N cumulative scores; their node indices in
 *   ASCENDING order (parents before children when nodes are numbered in the
 *   order they were drafted).  Equal scores go to the lower index.
 *     cum      [N] fp32, device;  1 <= N <= VT_TREE_MAX_CANDIDATES
 *     T        1 <= T <= min(N, VT_TREE_MAX_KEEP)
 *     out_idx  [T] int32, device, out
 *
 * Neither call needs a workspace; both enqueue one small kernel on `stream`.
 * ---------------------------------------------------------------------- */
#define VT_TREE_MAX_CANDIDATES 16384
#define VT_TREE_MAX_KEEP 1024
int vt_tree_expand(const float *parent_cum, const float *step_logp, const int32_t *step_ids, int32_t n,
                   int32_t m, int32_t K, int32_t *out_parent, int32_t *out_token, float *out_cum,
                   void *stream);
int vt_tree_rerank(const float *cum, int32_t N, int32_t T, int32_t *out_idx, void *stream);

/* ------------------------------------------------------------------------
 * vt_draft_tree_level -- one level of tree drafting in one call: the draft
 * step for the n frontier nodes followed by vt_tree_expand on its result,
 * with the same outputs as the two calls (bit for bit).  Where one kernel of
 * the step sees every row's result (always for n <= 8; up to 64 rows and
 * n * m <= 512 on the bf16 matrix-core path) no launch is added: the
 * workgroup that finishes the step last also ranks the n * m candidates;
 * other shapes run the step and then the expansion kernel.
 *   arguments as in vt_draft_head_step (no out_lse / out_logp_full) and
 *   vt_tree_expand; out_ids / out_logp [n, m] still receive the step's result.
 *   ws: >= vt_draft_head_step_ws_bytes(n, k, d, m); no initialisation.
 * ---------------------------------------------------------------------- */
int vt_draft_tree_level(const void *h, int h_type, int32_t n, const void *W_trim, int w_type, int32_t k,
                        int32_t d, const int32_t *map, int32_t m, const float *parent_cum, int32_t K,
                        int32_t *out_parent, int32_t *out_token, float *out_cum, int32_t *out_ids,
                        float *out_logp, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* VOCABTRIM_H_ */
