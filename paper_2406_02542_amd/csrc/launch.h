// Host-side launch interface between the C ABI (api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace loki {

constexpr int kD = 128;  // head dimension the kernels are written for

// Per-sequence sizes of a ragged batch, in device memory (a null pointer: the batch-wide value).
struct Ragged {
  const int32_t* seq_lens = nullptr;  // [B] cached rows of each sequence, 1..S
  const int32_t* ks = nullptr;        // [B] rows each sequence keeps, 1..min(k, its seq_len)
  int queries = 1;  // consecutive batch entries that share one cached sequence (several new
                    // tokens per sequence: entry b reads and appends to the cache of b / queries)
};

// The current token's key and value when the step also appends them to the cache (Algorithm 1
// lines 3-4 folded into the decode launch); both null otherwise.
struct Append {
  const void* k_new = nullptr;  // [B, Hkv, 128] unrotated key, storage type
  const void* v_new = nullptr;  // [B, Hkv, 128]
};

// A paged cache (table null: the contiguous layout [B, Hkv, S_cap, width]).  The three slabs
// are pools [n_pages, Hkv, page_rows, width]; row s of sequence b lives in physical page
// table[b * pages_per_seq + s / page_rows] at row s % page_rows, the same page for klo, khi, v.
struct Paging {
  const int32_t* table = nullptr;  // device [B, pages_per_seq]
  int lg_rows = 0;                 // log2(page_rows); page_rows is a power of two >= 256
  int pages_per_seq = 0;
  int n_pages = 0;                 // physical pages in the pools: table entries are clamped to it
};

struct Shape {
  int B, Hq, Hkv, G;  // G = Hq / Hkv
  int S, S_cap;       // S, k: the largest of the batch when `rg` gives per-sequence values
  int d, k;
  int dtype;        // 0 f32, 1 bf16
  int elem_bytes;   // 4 or 2
  Ragged rg;
  Append ap;
  Paging pg;
};

// Grid-shaping decisions; pure functions of the shape so that workspace sizing (host only)
// and the launchers agree.
constexpr int kDefaultCUs = 256;          // MI355X; what grids are shaped for when no device can be asked
// Compute units of the calling thread's current device (asked once per device and remembered;
// kDefaultCUs when there is no device, e.g. a size query on a machine without a GPU).  Grid
// shapes and the workspace layout that follows from them are functions of the shape and of this.
int device_cus();

// Raises the dynamic-LDS limit of a kernel the first time it is launched on each device (the
// attribute belongs to the function on one device; `done` is a bit mask of devices, one static
// per kernel instantiation, so that the launch path makes no attribute call afterwards).
hipError_t allow_dynamic_lds(const void* kernel, int bytes, std::atomic<unsigned long long>& done);
constexpr int kScoreRowsPerStep = 256;   // rows one 256-thread block scores per step
constexpr int kMaxGatherChunk = 2048;    // selected rows one attend block may own (LDS index list)
constexpr int kFusedMaxS = 8192;         // fused single-kernel path: scores of a unit live in LDS
constexpr int kFusedMaxK = 2048;

int score_rows_per_block(const Shape& s);
int gather_splits(const Shape& s, int select_mode);
int dense_splits(const Shape& s);

struct Workspace {
  float* qhat;       // [B*Hq, 128]
  float* scores;     // [B*Hsel, S]
  int32_t* sel_idx;  // [B*Hsel, k]
  float* sel_score;  // [B*Hsel, k] approximate scores of the selected rows
  int32_t* tickets;  // [B*Hq] finished row splits per head group; directly before sel_scratch, so
                     // that the rotation kernel clears it and the chunk histograms in one range
  size_t ticket_words;    // its padded length in words
  uint32_t* sel_scratch;  // long sequences only: chunk histograms, candidates, bookkeeping
  float* partial;    // [B*Hq, nsplit, 130]
  uint32_t* cluster_ctl;  // first bytes of every Loki workspace (kClusterCtlBytes): the arrival flags and tickets
                          // of the several-blocks-per-unit launch, at the same place whatever the shape
  void* cluster;     // exchange area of the several-blocks-per-unit launch (fused_gqa_cluster.hip), or null
  size_t total_bytes;
};
// Lays the workspace out from `base` (may be null to only size it).  with_cluster = false leaves
// the cluster launch's exchange area out (a workspace sized for a larger batch, which has no
// such area, still serves the other kernel sequences).
Workspace plan_workspace(const Shape& s, int select_mode, int nsplit, void* base, bool with_cluster = true);

// Rotates every query; with s.ap set also rotates the new key of every unit and writes it and
// the new value into row seq_len-1 of the unit's cache.
// zero_words / n_zero: words the kernel also clears (the gather's tickets and the chunk
// histograms of a long-sequence selection, which the score kernel then adds into); null: nothing.
hipError_t launch_qrot(const Shape& s, const void* q, const float* P, float* qhat, void* klo,
                       void* khi, void* v, uint32_t* zero_words, size_t n_zero, hipStream_t st);
// hist_part [selecting heads][hist_chunks][2048] (zeroed) or null: see select_hist_chunks.
hipError_t launch_score(const Shape& s, int select_mode, const void* q, const float* P,
                        const void* klo, float* scores, float* qhat, uint32_t* hist_part,
                        int hist_chunks, hipStream_t st);
size_t select_scratch_words(int S, int n_sel_heads);
// Long sequences, one token per sequence: the number of 16384-row chunks whose leading-digit
// histograms the score kernel fills for the selection (they are the first words of the select
// scratch), 0 when the selection counts for itself.
int select_hist_chunks(const Shape& s, int select_mode);
// sel_idx / sel_score: the selection.  one_pass (the score kernel filled the chunk histograms,
// select_hist_chunks != 0): the list is left as two ascending runs, the certain rows and then
// the chosen candidates, and only then: user_idx (nullable): the caller's ascending copy.
hipError_t launch_select(const Shape& s, int n_sel_heads, const float* scores, int32_t* sel_idx,
                         float* sel_score, uint32_t* scratch, bool one_pass, int32_t* user_idx,
                         hipStream_t st);
// tickets [B*Hq] (zeroed, see launch_qrot) or null: with more than one row split, the block that
// finishes a head group last merges the splits and writes `out`; null leaves the partials for
// launch_combine.
hipError_t launch_gather(const Shape& s, int select_mode, int nsplit, const float* qhat,
                         const void* klo, const void* khi, const void* v, const int32_t* sel_idx,
                         const float* sel_score, float* partial, int32_t* tickets, void* out,
                         hipStream_t st);
hipError_t launch_dense(const Shape& s, int nsplit, const void* q, const void* k_full,
                        const void* v, float* partial, void* out, hipStream_t st);
// Matrix-core attention for 8 query heads per block on bf16 caches (attend_mfma.hip).
bool attend_mfma_applies(const Shape& s, int heads_per_block);
hipError_t launch_dense_mfma(const Shape& s, int nsplit, const void* q, const void* k_full,
                             const void* v, float* partial, void* out, hipStream_t st);
hipError_t launch_pca_mfma(const Shape& s, int nsplit, const float* qhat, const void* klo,
                           const void* v, float* partial, void* out, hipStream_t st);
hipError_t launch_gather_mfma(const Shape& s, int nsplit, const float* qhat, const void* klo,
                              const void* khi, const void* v, const int32_t* sel_idx, float* partial,
                              int32_t* tickets, void* out, hipStream_t st);
// Appendix E, Algorithm 2: every row, logits from the low-rank slab alone.
hipError_t launch_pca_attend(const Shape& s, int nsplit, const float* qhat, const void* klo,
                             const void* v, float* partial, void* out, hipStream_t st);
hipError_t launch_combine(const Shape& s, int nsplit, const float* partial, void* out,
                          hipStream_t st);
// Fused single-kernel decode step (one query head per KV head only).
bool fused_eligible(const Shape& s);
bool fused_preferred(const Shape& s);
hipError_t launch_fused(const Shape& s, const void* q, const float* P, void* klo, void* khi,
                        void* v, void* out, int32_t* out_idx, hipStream_t st);
// Single-launch step for grouped query heads sharing one selection per KV head (fused_gqa.hip;
// bf16 caches, select_mode = one selection per KV group).
bool fused_gqa_eligible(const Shape& s, int select_mode);
bool fused_gqa_preferred(const Shape& s, int select_mode);
hipError_t launch_fused_gqa(const Shape& s, const void* q, const float* P, const void* klo,
                            const void* khi, const void* v, void* out, int32_t* out_idx,
                            hipStream_t st);
// The same step with 2, 4 or 8 cooperating blocks per unit, for launches with fewer units than
// compute units (fused_gqa_cluster.hip).  fused_gqa_cluster_blocks: blocks per unit the shape
// would get (0: not applicable; a function of B, Hkv, G, d, S, k and the device alone, so that
// the workspace can be sized without the step's other arguments); `region`: the workspace's
// exchange area of fused_gqa_cluster_bytes bytes.
int fused_gqa_cluster_blocks(const Shape& s, int select_mode);
size_t fused_gqa_cluster_bytes(const Shape& s, int select_mode);
bool fused_gqa_cluster_eligible(const Shape& s, int select_mode);
bool fused_gqa_cluster_preferred(const Shape& s, int select_mode);
// Polls a block of a cluster spends in one wait before it gives up (a test aid: the default is
// seconds; nothing a wait is for takes longer than the launch itself).
constexpr uint32_t kClusterSpinLimit = 1u << 22;
constexpr int kClusterMax = 8;             // blocks per unit at most
constexpr int kClusterMaxUnits = 128;      // units of a cluster launch at most (two blocks each on 256 compute units)
constexpr int kClusterFlagStride = 16;     // words between the arrival flags of two blocks: a cache line each
constexpr int kClusterCounterStride = (kClusterMax + 1) * kClusterFlagStride;  // words of a unit's flags and ticket
// the control words of every unit a cluster launch can have, and the error word behind them
constexpr size_t kClusterCtlBytes = ((size_t)kClusterMaxUnits * kClusterCounterStride + 64) * 4;
void set_cluster_spin_limit(uint32_t polls);
// ctl: the workspace's control words (Workspace::cluster_ctl); ctl_clean: they are known to be
// zero (a workspace the caller cleared once and only this library has written since: every
// finished launch leaves them zero), so no clearing kernel goes in front.
hipError_t launch_fused_gqa_cluster(const Shape& s, const void* q, const float* P, const void* klo,
                                    const void* khi, const void* v, void* out, int32_t* out_idx,
                                    uint32_t* ctl, bool ctl_clean, void* region, hipStream_t st);
// Calibration and diagnostics (calibrate.hip).
size_t pca_workspace_bytes(int Hkv, long long N);
hipError_t launch_pca_stage(int stage, int Hkv, int dtype, const void* keys, long long N, float* P,
                            float* eigenvalues, void* workspace, hipStream_t st);
hipError_t launch_rank_at(const float* eigenvalues, int n, int Dn, float v_percent, int32_t* ranks,
                          hipStream_t st);
hipError_t launch_layer_width(const float* eigenvalues, int n, int Dn, float v_percent, int multiple,
                              float* mean_rank, int32_t* d_out, hipStream_t st);
hipError_t launch_jaccard(const int32_t* a, const int32_t* b, int n_lists, int k, float* out,
                          hipStream_t st);
hipError_t launch_rotate(const Shape& s, const void* k_new, const float* P, void* klo, void* khi,
                         int pos, int n_new, hipStream_t st);

}  // namespace loki
