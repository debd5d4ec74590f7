/*
 * loki.h — C ABI of the MI355X (gfx950) Loki decode-attention library.
 *
 * Loki (arXiv 2406.02542) speeds up the decode step of attention: the key cache
 * holds keys rotated into a fixed PCA basis P (Khat = K P); per step the query
 * is rotated (qhat = q P), approximate scores are taken against the first d
 * columns of Khat only, the k best-scoring tokens are selected, and exact
 * softmax attention runs over those k rows in the rotated space (Algorithm 1,
 * Section 4.2; exactness of the rotated scores is Lemma 4.1).
 *
 * Conventions common to every call
 *   - All data pointers are DEVICE pointers unless marked "host".  `stream` is a
 *     hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work on `stream` and return without synchronising.
 *   - The caller owns every buffer, including the workspace.  The library
 *     allocates no device memory and keeps no state between calls beyond
 *     per-device facts it establishes once (the number of compute units, which
 *     shapes grids and workspace layouts; the address of the built-in buffer of
 *     loki_decode_attn_static; that a kernel's shared-memory limit has been
 *     raised on the device); calls on different streams with different
 *     workspaces may overlap.  Size a workspace with the device it will be used
 *     on current.
 *   - Every entry point returns a loki_status.  Arguments are validated on the
 *     host before anything is launched; on any non-zero status nothing was
 *     enqueued, except LOKI_ERR_HIP, which reports a launch error.
 *   - Head dimension D must be 128.  Storage type is fp32 or bf16 for q, the
 *     caches and the output; P is always fp32; all accumulation is fp32 and the
 *     output is rounded once (nearest-even) to the storage type.
 *   - NaN or Inf in the inputs: behaviour unspecified.
 *
 * Cache layout (per batch b and KV head h; S_cap rows are allocated, S are live)
 *     klo [B, Hkv, S_cap, d_split]       first d_split columns of Khat
 *     khi [B, Hkv, S_cap, D - d_split]   remaining columns of Khat
 *     v   [B, Hkv, S_cap, D]             values, not rotated
 *   Together klo and khi hold each rotated key exactly once (Section 4.2:
 *   the cache is no larger than the original one, plus P).  d_split must be a
 *   multiple of 16 bytes / element size; base pointers must be 16-byte aligned.
 *   khi is unused (may be NULL) when d_split == D.
 *
 * Projection P [Hkv, D, D], row-major, fp32: qhat_j = sum_i q_i P[h][i][j]; the
 * columns are the principal components, most important first.  Query head hq
 * uses KV head hq / (Hq / Hkv).
 */
#ifndef LOKI_H
#define LOKI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LOKI_OK = 0,
  LOKI_ERR_INVALID_ARG = 1,     /* null pointer, size out of range, Hq % Hkv != 0 ...   */
  LOKI_ERR_UNSUPPORTED = 2,     /* D != 128, unknown dtype, d not loadable in 16-B units,
                                   Hq / Hkv not in {1, 2, 4, 8}, B * Hq > 65535           */
  LOKI_ERR_ALIGNMENT = 3,       /* a base pointer is not 16-byte aligned                  */
  LOKI_ERR_WORKSPACE = 4,       /* workspace smaller than loki_workspace_bytes reports    */
  LOKI_ERR_HIP = 5,             /* the HIP runtime reported an error at launch            */
  LOKI_ERR_SCRATCH_LIMIT = 6    /* loki_decode_attn_static: the shape needs more workspace
                                   than LOKI_STATIC_SCRATCH_BYTES                         */
} loki_status;

enum { LOKI_F32 = 0, LOKI_BF16 = 1 };

/* How the k rows are chosen when several query heads share a KV head (the paper's
 * Algorithm 1 is written for one query head and does not treat grouped queries).
 *   PER_QUERY_HEAD: each query head ranks and picks its own k rows (literal reading).
 *   PER_KV_GROUP:   one set per KV head, ranked by the maximum over the group's
 *                   approximate scores; every query head of the group attends over it.
 * Both are identical when Hq == Hkv. */
enum { LOKI_SELECT_PER_QUERY_HEAD = 0, LOKI_SELECT_PER_KV_GROUP = 1 };

/* Optional bits OR-ed into select_mode that pin the kernel sequence (for tests and
 * benchmarks; by default the library chooses).  SPLIT: separate score, select and attention
 * kernels with the work of a unit spread over many blocks.  FUSED: one kernel, one block per
 * unit; available when Hq == Hkv, S <= 8192 and k <= 2048, and for grouped heads
 * (Hq / Hkv in {2, 4, 8}) with LOKI_SELECT_PER_KV_GROUP on a bf16 cache with d in {16, 32, 64},
 * S <= 16384, k <= 2048 (per-sequence lengths, the append and a paged cache of at most 64
 * pages per sequence of loki_decode_step included), one token per sequence (else
 * LOKI_ERR_UNSUPPORTED).  CLUSTER: the grouped-heads kernel of FUSED with 2, 4 or 8 cooperating
 * blocks per (batch, KV head) unit, each on a slice of the unit's rows, for batches with too few
 * units to fill the chip with one block each: the same conditions as FUSED for grouped heads
 * except that B * Hkv (rounded up to a multiple of 8) is at most half the device's compute units
 * (and at most 128),
 * and S / blocks <= 16384, min(k, S / blocks) <= 8192 (so S up to 131072 and k up to 8192 with
 * 8 blocks).  Its blocks wait for each other inside the
 * launch: every wait is bounded, and a block that gives up (see loki_debug_cluster_spin_limit)
 * writes NaN into its unit's outputs.  All three give the same selected sets; outputs agree
 * to fp32 rounding (bf16 rounding of two-term products for grouped heads). */
enum { LOKI_PATH_SPLIT = 0x100, LOKI_PATH_FUSED = 0x200, LOKI_PATH_CLUSTER = 0x300, LOKI_PATH_MASK = 0x300 };

/* Optional bit OR-ed into select_mode: the caller vouches that the workspace was filled with
 * zeros after it was allocated and that nothing but calls of this library (any shapes) has
 * written to it since.  LOKI_PATH_CLUSTER keeps a few control words at the start of the
 * workspace that must be zero when a launch starts; every finished launch leaves them zero, so
 * with this bit the clearing kernel in front of the launch (about 5 us) is left out.  Without the
 * bit the workspace needs no initialisation at all.  A launch whose blocks gave up waiting
 * (NaN outputs) leaves a mark there: with the bit, later LOKI_PATH_CLUSTER launches on that
 * workspace write NaN too until it is filled with zeros again. */
enum { LOKI_WORKSPACE_ZEROED = 0x400 };

typedef struct {
  int32_t B;        /* sequences in the batch; B * Hq <= 65535           */
  int32_t Hq;       /* query heads                                    */
  int32_t Hkv;      /* KV heads; Hq % Hkv == 0                        */
  int32_t D;        /* head dimension (128)                           */
  int32_t d_split;  /* columns of Khat kept in the low-rank slab klo  */
  int32_t S_cap;    /* rows allocated per (b, h) in klo / khi / v     */
  int32_t dtype;    /* LOKI_F32 or LOKI_BF16                          */
} loki_layout;

/* Library version, major*10000 + minor*100 + patch. */
int loki_version(void);

/* Static, human-readable name of a status code (host pointer, never NULL). */
const char* loki_status_string(int status);

/* Bytes of the three cache arrays for a layout.  Host-only; touches no GPU. */
int loki_cache_bytes(const loki_layout* layout, size_t* klo_bytes, size_t* khi_bytes,
                     size_t* v_bytes);

/* Bytes of workspace loki_decode_attn needs for (S, d, k, select_mode) and
 * dense_decode_attn needs for S (pass d = 0, k = 0, select_mode = -1 for the
 * dense baseline).  Host-only; touches no GPU.  The workspace holds the
 * approximate scores, the selected indices, qhat, the partial softmax
 * results of split rows and, for shapes that LOKI_PATH_CLUSTER takes, the area
 * its blocks exchange counts through; its contents are undefined between calls
 * and nothing in it has to be initialised.  A workspace sized for a larger
 * batch of the same layout also serves a smaller one (without room for the
 * exchange area the library picks another kernel sequence; LOKI_PATH_CLUSTER
 * pinned then returns LOKI_ERR_WORKSPACE). */
int loki_workspace_bytes(const loki_layout* layout, int S, int d, int k, int select_mode,
                         size_t* bytes);

/*
 * Algorithm 1 lines 3-4: rotate n_new new keys per (b, h) into the PCA basis and
 * store them in the cache, khat = k P_h, rounded to the storage type.
 *   k_new [B, Hkv, n_new, D]  keys in the model's basis (storage type)
 *   P     [Hkv, D, D]         fp32
 *   klo, khi                  cache slabs; rows [pos, pos + n_new) of every (b, h)
 *                             are overwritten, other rows are untouched
 * Requires 0 <= pos, 1 <= n_new, pos + n_new <= S_cap.  Values are appended by the
 * caller directly (V is not transformed).
 */
int loki_rotate_keys(const loki_layout* layout, const void* k_new, const float* P, void* klo,
                     void* khi, int pos, int n_new, void* stream);

/*
 * loki_rotate_keys into a paged cache (see loki_decode_step for the page table's meaning):
 * klo and khi are the pools [n_pages, Hkv, page_rows, d | D - d]; rows pos .. pos + n_new - 1
 * of every sequence go to the pages page_table[b, row / page_rows] names;
 * pages_per_seq * page_rows >= pos + n_new, which also has to fit layout->S_cap.  V is not
 * transformed and is written by the caller.
 */
int loki_rotate_keys_paged(const loki_layout* layout, const void* k_new, const float* P, void* klo,
                           void* khi, const int32_t* page_table, int page_rows, int pages_per_seq,
                           int n_pages, int pos, int n_new, void* stream);

/*
 * Algorithm 1 lines 3 and 5-9 for every (b, query head): the decode step.
 *   q    [B, Hq, D]   queries in the model's basis (storage type)
 *   P    [Hkv, D, D]  fp32
 *   klo, khi, v       the cache; rows [0, S) are read
 *   S                 live rows, 1 <= S <= S_cap (the new token's key is already
 *                     in the cache and competes like any other row)
 *   d                 ranking columns; must equal layout->d_split
 *   k                 rows kept, 1 <= k <= S
 *   select_mode       LOKI_SELECT_*
 *   workspace         >= loki_workspace_bytes(layout, S, d, k, select_mode), 256-B aligned
 *   out  [B, Hq, D]   softmax(qhat Khat'^T / sqrt(D)) V' over the selected rows
 *                     (storage type)
 *   out_idx           NULL, or int32 [B, Hsel, k] (Hsel = Hq or Hkv by select_mode):
 *                     receives the selected positions in ascending order.  Ranking is
 *                     by signed value of the unscaled approximate score computed in
 *                     fp32; among equal scores the lowest position is kept.
 */
int loki_decode_attn(const loki_layout* layout, const void* q, const float* P, const void* klo,
                     const void* khi, const void* v, int S, int d, int k, int select_mode,
                     void* workspace, size_t workspace_bytes, void* out, int32_t* out_idx,
                     void* stream);

/*
 * loki_decode_attn for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * scores, index lists, rotated queries and split partials go to a buffer of
 * LOKI_STATIC_SCRATCH_BYTES that is part of the library's device image (one copy per GPU, held
 * until the process ends); the call allocates and frees nothing.  Arguments and results as
 * loki_decode_attn, without workspace / workspace_bytes.
 *   - A shape whose loki_workspace_bytes(layout, S, d, k, select_mode) exceeds
 *     LOKI_STATIC_SCRATCH_BYTES is refused with LOKI_ERR_SCRATCH_LIMIT; nothing is enqueued.
 *   - The device the work runs on must be the calling thread's current device.  The first call
 *     on a device looks the buffer's address up (hipGetSymbolAddress); make that call before
 *     starting a graph capture.
 *   - All calls on one GPU share that GPU's buffer, which keeps the previous call's contents
 *     (no kernel relies on them; nothing has to be cleared).  Calls that may run at the same
 *     time on one GPU (different streams) race on it: serialise them, or use loki_decode_attn
 *     with separate workspaces.
 */
enum { LOKI_STATIC_SCRATCH_BYTES = 64 << 20 };
int loki_decode_attn_static(const loki_layout* layout, const void* q, const float* P,
                            const void* klo, const void* khi, const void* v, int S, int d, int k,
                            int select_mode, void* out, int32_t* out_idx, void* stream);

/*
 * Section 2, Eq. 1: full attention over all S rows, the baseline Loki is compared
 * with.  Works on an unsplit key cache.
 *   q      [B, Hq, D]
 *   k_full [B, Hkv, S_cap, D]   keys (any basis consistent with q; storage type)
 *   v      [B, Hkv, S_cap, D]
 *   out    [B, Hq, D]           softmax(q K^T / sqrt(D)) V
 * layout->d_split is ignored.  Query heads of a group share one pass over K and V.
 */
int dense_decode_attn(const loki_layout* layout, const void* q, const void* k_full, const void* v,
                      int S, void* workspace, size_t workspace_bytes, void* out, void* stream);

/*
 * The whole decode step of Algorithm 1 (lines 2-9) for a batch whose sequences may
 * differ in length, optionally including the cache append of the current token
 * (lines 3-4: rotate the new key, store it and the new value), in the same launches
 * as the attention.  With args == NULL, or all of its members NULL, it is
 * loki_decode_attn.
 *
 *   seq_lens  device int32 [B] or NULL: rows sequence b holds, counting the current
 *             token, 1 <= seq_lens[b] <= S_max.  NULL: S_max for every sequence.
 *   ks        device int32 [B] or NULL: rows sequence b keeps,
 *             1 <= ks[b] <= min(k_max, seq_lens[b]).  NULL: min(k_max, seq_lens[b]).
 *             Entries outside their range are clamped into it.
 *   k_new     device [B, Hkv, D] or NULL: unrotated key of the current token (storage
 *             type).  When given, Khat row seq_lens[b]-1 of every (b, KV head) is
 *             overwritten with round(k_new P_h) (columns < d into klo, the rest into
 *             khi, as loki_rotate_keys does) and V row seq_lens[b]-1 with v_new, before
 *             anything is scored; the step then sees them like any cached row.
 *   v_new     device [B, Hkv, D]; required exactly when k_new is given.
 *
 *   queries_per_seq  m; 0 or 1: one new token per sequence.  m > 1 (chunked or speculative
 *             decoding): the last m tokens of every sequence are decoded at once.  Every
 *             per-sequence argument then has m consecutive entries per sequence, token j of
 *             sequence b at entry b m + j: q, out [B, m, Hq, D]; out_idx [B, m, Hsel, k_max];
 *             k_new, v_new [B, m, Hkv, D]; seq_lens, ks [B m], seq_lens required, with
 *             seq_lens[b m + j] = rows token j may see, counting itself (the causal limit:
 *             normally rows_b - (m - 1 - j)).  Entry b m + j appends to row
 *             seq_lens[b m + j] - 1 of sequence b's cache; all m rows are written before
 *             anything is scored.  The workspace is sized for a layout with B m in place of B.
 *
 *   page_table  device int32 [B, pages_per_seq] or NULL.  When given, the cache is paged:
 *             klo, khi and v are pools [n_pages, Hkv, page_rows, d | D - d | D] and row s of
 *             sequence b lives in physical page page_table[b * pages_per_seq + s / page_rows]
 *             at row s % page_rows, the same page of all three pools.  page_rows is a power of
 *             two >= 256; pages_per_seq * page_rows >= S_max; entries are clamped into
 *             [0, n_pages); n_pages * Hkv * page_rows < 2^31.  layout->S_cap is then only the
 *             bound of S_max.
 *
 * S_max and k_max (1 <= k_max <= S_max <= S_cap) size the workspace
 * (loki_workspace_bytes(layout, S_max, d, k_max, select_mode)) and out_idx:
 * out_idx is [B, Hsel, k_max], and a sequence keeping fewer than k_max rows has -1 in
 * the remaining entries.  klo, khi and v are written only when k_new is given.
 * Everything else as loki_decode_attn.
 */
typedef struct {
  const int32_t* seq_lens;
  const int32_t* ks;
  const void* k_new;
  const void* v_new;
  int32_t queries_per_seq;
  int32_t page_rows;
  const int32_t* page_table;
  int32_t pages_per_seq;
  int32_t n_pages;
} loki_step_args;

int loki_decode_step(const loki_layout* layout, const void* q, const float* P, void* klo, void* khi,
                     void* v, int S_max, int d, int k_max, int select_mode,
                     const loki_step_args* args, void* workspace, size_t workspace_bytes, void* out,
                     int32_t* out_idx, void* stream);

/*
 * dense_decode_attn with per-sequence lengths: sequence b attends over its first
 * seq_lens[b] rows (device int32 [B], 1 <= seq_lens[b] <= S_max; NULL: S_max).  The
 * workspace is sized for S_max (loki_workspace_bytes(layout, S_max, 0, 0, -1)).
 */
int dense_decode_step(const loki_layout* layout, const void* q, const void* k_full, const void* v,
                      int S_max, const int32_t* seq_lens, void* workspace, size_t workspace_bytes,
                      void* out, void* stream);

/*
 * Appendix E, Algorithm 2 (PCAAttn, the variant the paper tried and set aside): the
 * attention weights come from the first d rotated columns alone, over all S rows,
 *   out = softmax(qhat[:d] Klo^T / sqrt(D)) V,
 * so only the low-rank slab of the key cache is read (with d = D it is Eq. 1 in the
 * rotated basis).  Arguments as loki_decode_attn; the workspace holds the rotated
 * queries and split partials: loki_workspace_bytes(layout, S, d, 0, -2).
 */
int loki_pca_attn(const loki_layout* layout, const void* q, const float* P, const void* klo,
                  const void* v, int S, int d, void* workspace, size_t workspace_bytes, void* out,
                  void* stream);

/*
 * Section 3.1: the PCA of a set of calibration keys that produces the basis P.
 *   keys        [Hkv, n_rows, D] device, storage type of layout->dtype (layout's B,
 *               Hq, S_cap and d_split are not used)
 *   P           [Hkv, D, D] fp32 out: column j = j-th principal component (eigenvector of
 *               the sample covariance of the head's keys, mean removed), decreasing
 *               eigenvalue; the largest-magnitude entry of every column is positive
 *   eigenvalues [Hkv, D] fp32 out, decreasing
 *   workspace   >= loki_pca_workspace_bytes(layout, n_rows), 256-B aligned
 * Covariance: matrix cores with fp32 accumulation per run of rows, runs added in fp64;
 * eigensolver: cyclic Jacobi in fp64.  2 <= n_rows.
 */
int loki_pca_workspace_bytes(const loki_layout* layout, long long n_rows, size_t* bytes);
int loki_pca_fit(const loki_layout* layout, const void* keys, long long n_rows, float* P,
                 float* eigenvalues, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Section 3.1, Eq. 2 (Rank@v): for each of n_heads spectra (device fp32 [n_heads, D],
 * decreasing), the smallest d whose first d eigenvalues hold at least v_percent per cent
 * of the total; ranks is device int32 [n_heads].  0 < v_percent <= 100.
 */
int loki_rank_at(const float* eigenvalues, int n_heads, int D, float v_percent, int32_t* ranks,
                 void* stream);

/*
 * Section 3.1 (Rank_l@v: Rank_{l,h}@v of Eq. 2 averaged over the heads of a layer) and
 * Appendix B.2 (a layer's slab width set from its explained variance).  eigenvalues is
 * device fp32 [n_heads, D], decreasing per head.  mean_rank (device fp32 [1], may be NULL)
 * receives Rank_l@v; d_out (device int32 [1]) receives the width: Rank_l@v taken up to the
 * next whole number, then up to the next multiple of `multiple` (the layout's granularity:
 * 8 for bf16 caches, 4 for fp32; D % multiple == 0), at most D.  0 < v_percent <= 100.
 * The value is what loki_layout.d_split of that layer's cache would be set to; the caller
 * reads it back.  Errors as for loki_rank_at.
 */
int loki_layer_width(const float* eigenvalues, int n_heads, int D, float v_percent, int multiple,
                     float* mean_rank, int32_t* d_out, void* stream);

/*
 * Section 6.3 (agreement of two selections, Figure 6 left): Jaccard similarity
 * |A n B| / |A u B| of n_lists pairs of ascending index lists (device int32
 * [n_lists, k], entries < 0 are padding at the end); out is device fp32 [n_lists].
 */
int loki_index_jaccard(const int32_t* idx_a, const int32_t* idx_b, int n_lists, int k, float* out,
                       void* stream);

/*
 * Stage timing for benchmarks.  A profile owns HIP events; when one is attached
 * with loki_profile_attach, the next decode / dense / rotate calls made from the
 * same host thread record an event before and after every kernel they launch (on
 * the call's stream).  loki_profile_read synchronises on the last event and
 * returns, for the most recent call, the number of kernels and the elapsed
 * milliseconds of each (ms[i] for the i-th kernel, in launch order; names[i]
 * points at a static string).  Detach with loki_profile_attach(NULL).
 */
typedef struct loki_profile loki_profile;
enum { LOKI_PROFILE_MAX_KERNELS = 8 };
int loki_profile_create(loki_profile** out);
int loki_profile_destroy(loki_profile* p);
int loki_profile_attach(loki_profile* p);
int loki_profile_read(loki_profile* p, int* n_kernels, float* ms, const char** names);

/*
 * Test aid for LOKI_PATH_CLUSTER, whose blocks wait for each other: the number of polls a block
 * spends in one wait before it gives up, raises the error state and writes NaN into the outputs
 * of its unit (the default, restored by 0, is a few seconds' worth; a wait normally ends within
 * microseconds).  With a limit of 1 a test can watch the give-up path: the launch still ends and
 * every output is either right or NaN.  Process-wide; affects launches enqueued afterwards.
 */
int loki_debug_cluster_spin_limit(unsigned polls);

/*
 * Whether a LOKI_PATH_CLUSTER launch on this workspace gave up waiting since its control words
 * were last cleared (by the clearing kernel in front of every launch without
 * LOKI_WORKSPACE_ZEROED, else by the caller's zero fill): *gave_up = 1 or 0 (host pointer).
 * Copies one word from the workspace after everything enqueued on `stream` so far has finished;
 * returns when the answer is there.  `workspace` as passed to the decode call.
 */
int loki_cluster_gave_up(const void* workspace, int* gave_up, void* stream);

/*
 * Measurement aid, not part of the method: enqueues one trivial kernel that reads
 * `bytes` bytes (a multiple of 16, 16-byte aligned device pointer) with coalesced
 * 16-byte loads and discards them.  Its duration over as many bytes as a decode step
 * moves is the read ceiling a benchmark can set beside the published HBM peak.
 */
int loki_stream_read(const void* buf, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LOKI_H */
