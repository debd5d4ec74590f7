// C ABI of the Loki decode-attention library: argument validation, workspace planning and
// kernel sequencing.  See include/loki.h for the contract of every entry point.
#include "../../include/loki.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <new>

#include "launch.h"

namespace loki {

static inline int div_up(int a, int b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int device_cus() {
  constexpr int kSlots = 64;
  static std::atomic<int> cached[kSlots];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kSlots) {
    (void)hipGetLastError();  // a size query without a device is not an error of a later launch
    return kDefaultCUs;
  }
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
    (void)hipGetLastError();
    n = kDefaultCUs;
  }
  cached[dev].store(n, std::memory_order_relaxed);
  return n;
}

hipError_t allow_dynamic_lds(const void* kernel, int bytes, std::atomic<unsigned long long>& done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
  const unsigned long long bit = 1ull << (dev & 63);
  if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && dev < 64) done.fetch_or(bit, std::memory_order_release);
  return e;
}

int score_rows_per_block(const Shape& s) {
  const int units = s.B * s.Hkv;
#ifndef LOKI_SCORE_BLOCKS_PER_CU
#define LOKI_SCORE_BLOCKS_PER_CU 8
#endif
  int nchunks = div_up(LOKI_SCORE_BLOCKS_PER_CU * device_cus(), units);
  const int max_chunks = div_up(s.S, 2 * kScoreRowsPerStep);
  if (nchunks > max_chunks) nchunks = max_chunks;
  if (nchunks < 1) nchunks = 1;
  int rows = div_up(div_up(s.S, nchunks), kScoreRowsPerStep) * kScoreRowsPerStep;
  if (s.S > 16384) {
    // long sequences: a block stays inside one 16384-row chunk of the selection (it adds its
    // counts into that chunk's histogram): a power of two of at most 16384 rows
    int r = kScoreRowsPerStep;
    while (2 * r <= rows && 2 * r <= 16384) r *= 2;
    rows = r;
  }
  if (s.pg.table != nullptr) {
    // a block must lie inside one page: the largest power of two (>= 256) within rows and the page
    const int page_rows = 1 << s.pg.lg_rows;
    int r = kScoreRowsPerStep;
    while (2 * r <= rows && 2 * r <= page_rows) r *= 2;
    rows = r;
  }
  return rows;
}

int gather_splits(const Shape& s, int select_mode) {
  const int heads = (select_mode == 1) ? s.B * s.Hkv : s.B * s.Hq;
  // about two blocks per CU: a block's set-up and merge cost as much as a few hundred rows, and
  // a launch that needs no split also needs no combine kernel
  int n = div_up(2 * device_cus(), heads);
  const int max_n = s.k / 128 > 0 ? s.k / 128 : 1;
  if (n > max_n) n = max_n;
  const int min_n = div_up(s.k, kMaxGatherChunk);
  if (n < min_n) n = min_n;
  return n;
}

int dense_splits(const Shape& s) {
  const int units = s.B * s.Hkv;
  int n = div_up(8 * device_cus(), units);
  const int max_n = s.S / 256 > 0 ? s.S / 256 : 1;
  if (n > max_n) n = max_n;
  return n < 1 ? 1 : n;
}

Workspace plan_workspace(const Shape& s, int select_mode, int nsplit, void* base, bool with_cluster) {
  Workspace w{};
  char* p = static_cast<char*>(base);
  size_t off = 0;
  const size_t heads_q = (size_t)s.B * s.Hq;
  auto take = [&](size_t bytes) {
    char* r = p ? p + off : nullptr;
    off += align_up(bytes, 256);
    return r;
  };
  if (select_mode == -2) w.qhat = reinterpret_cast<float*>(take(heads_q * kD * sizeof(float)));
  if (select_mode >= 0) {
    const size_t heads_sel = (select_mode == 1) ? (size_t)s.B * s.Hkv : heads_q;
    w.cluster_ctl = reinterpret_cast<uint32_t*>(take(kClusterCtlBytes));  // at offset 0 for every shape
    w.qhat = reinterpret_cast<float*>(take(heads_q * kD * sizeof(float)));
    w.scores = reinterpret_cast<float*>(take(heads_sel * s.S * sizeof(float)));
    w.sel_idx = reinterpret_cast<int32_t*>(take(heads_sel * s.k * sizeof(int32_t)));
    w.sel_score = reinterpret_cast<float*>(take(heads_sel * s.k * sizeof(float)));
    w.ticket_words = align_up(heads_q * sizeof(int32_t), 256) / 4;
    w.tickets = reinterpret_cast<int32_t*>(take(w.ticket_words * 4));
    const size_t scratch_words = select_scratch_words(s.S, (int)heads_sel);
    w.sel_scratch = scratch_words ? reinterpret_cast<uint32_t*>(take(scratch_words * 4)) : nullptr;
    if (scratch_words && !p) w.sel_scratch = nullptr;
    const size_t cluster_bytes = with_cluster ? fused_gqa_cluster_bytes(s, select_mode) : 0;
    w.cluster = cluster_bytes ? take(cluster_bytes) : nullptr;
  }
  w.partial = reinterpret_cast<float*>(
      take(nsplit > 1 ? heads_q * nsplit * (size_t)(kD + 2) * sizeof(float) : 0));
  w.total_bytes = off;
  return w;
}

// ---- stage timing ---------------------------------------------------------------------
}  // namespace loki

struct loki_profile {
  hipEvent_t ev[2 * LOKI_PROFILE_MAX_KERNELS];
  const char* names[LOKI_PROFILE_MAX_KERNELS];
  int n;
};

namespace loki {

static thread_local loki_profile* t_profile = nullptr;

struct StageTimer {
  hipStream_t st;
  explicit StageTimer(hipStream_t s) : st(s) {
    if (t_profile) t_profile->n = 0;
  }
  void begin(const char* name) {
    loki_profile* p = t_profile;
    if (!p || p->n >= LOKI_PROFILE_MAX_KERNELS) return;
    p->names[p->n] = name;
    (void)hipEventRecord(p->ev[2 * p->n], st);
  }
  void end() {
    loki_profile* p = t_profile;
    if (!p || p->n >= LOKI_PROFILE_MAX_KERNELS) return;
    (void)hipEventRecord(p->ev[2 * p->n + 1], st);
    p->n++;
  }
};

static int check_layout(const loki_layout* L, Shape* s) {
  if (!L) return LOKI_ERR_INVALID_ARG;
  if (L->B < 1 || L->Hq < 1 || L->Hkv < 1 || L->S_cap < 1) return LOKI_ERR_INVALID_ARG;
  if (L->Hq % L->Hkv != 0) return LOKI_ERR_INVALID_ARG;
  if (L->dtype != LOKI_F32 && L->dtype != LOKI_BF16) return LOKI_ERR_UNSUPPORTED;
  if (L->D != 128) return LOKI_ERR_UNSUPPORTED;
  const int eb = L->dtype == LOKI_F32 ? 4 : 2;
  if (L->d_split < 1 || L->d_split > L->D) return LOKI_ERR_INVALID_ARG;
  if ((L->d_split * eb) % 16 != 0) return LOKI_ERR_UNSUPPORTED;
  const int G = L->Hq / L->Hkv;
  if (G != 1 && G != 2 && G != 4 && G != 8) return LOKI_ERR_UNSUPPORTED;
  // heads index the second grid dimension of several kernels (at most 65 535 blocks)
  if ((long long)L->B * L->Hq > 65535) return LOKI_ERR_UNSUPPORTED;
  s->B = L->B;
  s->Hq = L->Hq;
  s->Hkv = L->Hkv;
  s->G = G;
  s->S_cap = L->S_cap;
  s->S = 0;
  s->d = L->d_split;
  s->k = 0;
  s->dtype = L->dtype;
  s->elem_bytes = eb;
  return LOKI_OK;
}

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

// ---- built-in scratch for callers that cannot allocate (loki_decode_attn_static) -----------
// Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address is looked up once per device (with that device current) and kept, and only
// that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[LOKI_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static int static_scratch_address(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return LOKI_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return LOKI_ERR_UNSUPPORTED;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr)
      return LOKI_ERR_HIP;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // every thread finds the same address
  }
  *out = ptr;
  return LOKI_OK;
}

}  // namespace loki

using namespace loki;

// Measurement aid: streams `n16` 16-byte words through the load path and discards them.  The
// time of this kernel over as many bytes as a decode step moves is the practical ceiling of
// a read-bound kernel on the device it runs on.
namespace loki {
__device__ unsigned g_stream_read_sink;
__global__ __launch_bounds__(512) void stream_read_kernel(const uint4* __restrict__ p, size_t n16) {
  unsigned acc = 0;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = p[i + u * stride];
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const uint4 v = p[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9e3779b9u) g_stream_read_sink = acc;  // keeps the loads alive
}
}  // namespace loki

extern "C" {

int loki_version(void) { return 110; }

const char* loki_status_string(int status) {
  switch (status) {
    case LOKI_OK: return "ok";
    case LOKI_ERR_INVALID_ARG: return "invalid argument";
    case LOKI_ERR_UNSUPPORTED: return "unsupported configuration";
    case LOKI_ERR_ALIGNMENT: return "pointer not sufficiently aligned";
    case LOKI_ERR_WORKSPACE: return "workspace too small";
    case LOKI_ERR_HIP: return "HIP runtime error";
    case LOKI_ERR_SCRATCH_LIMIT: return "shape needs more than the built-in scratch buffer";
    default: return "unknown status";
  }
}

int loki_cache_bytes(const loki_layout* layout, size_t* klo_bytes, size_t* khi_bytes,
                     size_t* v_bytes) {
  Shape s;
  const int rc = check_layout(layout, &s);
  if (rc != LOKI_OK) return rc;
  if (!klo_bytes || !khi_bytes || !v_bytes) return LOKI_ERR_INVALID_ARG;
  const size_t rows = (size_t)s.B * s.Hkv * s.S_cap;
  *klo_bytes = rows * s.d * s.elem_bytes;
  *khi_bytes = rows * (128 - s.d) * s.elem_bytes;
  *v_bytes = rows * 128 * s.elem_bytes;
  return LOKI_OK;
}

int loki_workspace_bytes(const loki_layout* layout, int S, int d, int k, int select_mode,
                         size_t* bytes) {
  Shape s;
  const int rc = check_layout(layout, &s);
  if (rc != LOKI_OK) return rc;
  if (!bytes) return LOKI_ERR_INVALID_ARG;
  if (S < 1 || S > s.S_cap) return LOKI_ERR_INVALID_ARG;
  s.S = S;
  if (select_mode == -1 || select_mode == -2) {  // dense baseline; PCAAttn (rotated queries too)
    *bytes = plan_workspace(s, select_mode, dense_splits(s), nullptr).total_bytes;
    return LOKI_OK;
  }
  if (select_mode < 0) return LOKI_ERR_INVALID_ARG;
  select_mode &= ~(LOKI_PATH_MASK | LOKI_WORKSPACE_ZEROED);
  if (select_mode != LOKI_SELECT_PER_QUERY_HEAD && select_mode != LOKI_SELECT_PER_KV_GROUP)
    return LOKI_ERR_INVALID_ARG;
  if (d != s.d) return LOKI_ERR_UNSUPPORTED;
  if (k < 1 || k > S) return LOKI_ERR_INVALID_ARG;
  s.k = k;
  *bytes = plan_workspace(s, select_mode, gather_splits(s, select_mode), nullptr).total_bytes;
  return LOKI_OK;
}

static int paging_from_args(const int32_t* page_table, int page_rows, int pages_per_seq, int n_pages,
                            int Hkv, long long rows_needed, Paging* pg) {
  int lg = 0;
  while (lg < 31 && (1 << lg) < page_rows) ++lg;
  if (page_rows < 1 || (1 << lg) != page_rows) return LOKI_ERR_INVALID_ARG;
  if (lg < 8 || lg > 24 || pages_per_seq < 1 || n_pages < 1) return LOKI_ERR_INVALID_ARG;
  if ((long long)pages_per_seq * page_rows < rows_needed) return LOKI_ERR_INVALID_ARG;
  if ((long long)n_pages * Hkv * page_rows > 0x7fffffffLL) return LOKI_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(page_table) & 3u) return LOKI_ERR_ALIGNMENT;
  pg->table = page_table;
  pg->lg_rows = lg;
  pg->pages_per_seq = pages_per_seq;
  pg->n_pages = n_pages;
  return LOKI_OK;
}

static int rotate_impl(const loki_layout* layout, const void* k_new, const float* P, void* klo,
                       void* khi, int pos, int n_new, const Paging* pg, void* stream) {
  Shape s;
  const int rc = check_layout(layout, &s);
  if (rc != LOKI_OK) return rc;
  if (!k_new || !P || !klo) return LOKI_ERR_INVALID_ARG;
  if (s.d < 128 && !khi) return LOKI_ERR_INVALID_ARG;
  if (pos < 0 || n_new < 1 || (long long)pos + n_new > s.S_cap) return LOKI_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(P) || !aligned16(klo) || !aligned16(khi))
    return LOKI_ERR_ALIGNMENT;
  if (pg) s.pg = *pg;
  hipStream_t st = static_cast<hipStream_t>(stream);
  StageTimer tm(st);
  tm.begin("rotate_keys");
  const hipError_t e = launch_rotate(s, k_new, P, klo, khi, pos, n_new, st);
  tm.end();
  return e == hipSuccess ? LOKI_OK : LOKI_ERR_HIP;
}

int loki_rotate_keys(const loki_layout* layout, const void* k_new, const float* P, void* klo,
                     void* khi, int pos, int n_new, void* stream) {
  return rotate_impl(layout, k_new, P, klo, khi, pos, n_new, nullptr, stream);
}

int loki_rotate_keys_paged(const loki_layout* layout, const void* k_new, const float* P, void* klo,
                           void* khi, const int32_t* page_table, int page_rows, int pages_per_seq,
                           int n_pages, int pos, int n_new, void* stream) {
  if (!layout || !page_table) return LOKI_ERR_INVALID_ARG;
  if (pos < 0 || n_new < 1) return LOKI_ERR_INVALID_ARG;
  Paging pg;
  const int rc = paging_from_args(page_table, page_rows, pages_per_seq, n_pages, layout->Hkv,
                                  (long long)pos + n_new, &pg);
  if (rc != LOKI_OK) return rc;
  return rotate_impl(layout, k_new, P, klo, khi, pos, n_new, &pg, stream);
}

// The decode step behind loki_decode_attn (no per-sequence sizes, no append) and
// loki_decode_step.
static int decode_impl(const loki_layout* layout, const void* q, const float* P, void* klo, void* khi,
                       void* v, int S, int d, int k, int select_mode, const Ragged& rg,
                       const Append& ap, const Paging& pg, void* workspace, size_t workspace_bytes,
                       void* out, int32_t* out_idx, void* stream) {
  Shape s;
  const int rc = check_layout(layout, &s);
  if (rc != LOKI_OK) return rc;
  if (rg.queries < 1 || rg.queries > 64) return LOKI_ERR_INVALID_ARG;
  if (rg.queries > 1) {
    // every query of a sequence is a batch entry of its own from here on; the kernels map
    // entry b back to the cache of sequence b / queries
    if ((long long)s.B * rg.queries * s.Hq > 65535) return LOKI_ERR_UNSUPPORTED;
    if (rg.seq_lens == nullptr) return LOKI_ERR_INVALID_ARG;  // each query has its own causal length
    s.B *= rg.queries;
  }
  if (!q || !P || !klo || !v || !out || !workspace) return LOKI_ERR_INVALID_ARG;
  if (s.d < 128 && !khi) return LOKI_ERR_INVALID_ARG;
  const int path = select_mode & LOKI_PATH_MASK;
  const bool ws_zeroed = (select_mode & LOKI_WORKSPACE_ZEROED) != 0;
  select_mode &= ~(LOKI_PATH_MASK | LOKI_WORKSPACE_ZEROED);
  if (select_mode != LOKI_SELECT_PER_QUERY_HEAD && select_mode != LOKI_SELECT_PER_KV_GROUP)
    return LOKI_ERR_INVALID_ARG;
  if (path != 0 && path != LOKI_PATH_SPLIT && path != LOKI_PATH_FUSED && path != LOKI_PATH_CLUSTER)
    return LOKI_ERR_INVALID_ARG;
  if (S < 1 || S > s.S_cap) return LOKI_ERR_INVALID_ARG;
  if (k < 1 || k > S) return LOKI_ERR_INVALID_ARG;
  if (d != s.d) return LOKI_ERR_UNSUPPORTED;
  if ((ap.k_new == nullptr) != (ap.v_new == nullptr)) return LOKI_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(P) || !aligned16(klo) || !aligned16(khi) || !aligned16(v) ||
      !aligned16(out) || !aligned16(out_idx) || !aligned16(ap.k_new) || !aligned16(ap.v_new))
    return LOKI_ERR_ALIGNMENT;
  if ((reinterpret_cast<uintptr_t>(rg.seq_lens) & 3u) || (reinterpret_cast<uintptr_t>(rg.ks) & 3u))
    return LOKI_ERR_ALIGNMENT;
  if (!aligned256(workspace)) return LOKI_ERR_ALIGNMENT;
  s.S = S;
  s.k = k;
  s.rg = rg;
  s.ap = ap;
  s.pg = pg;
  if (s.G == 1) select_mode = LOKI_SELECT_PER_QUERY_HEAD;  // identical; one code path
  const int nsplit = gather_splits(s, select_mode);
  Workspace w = plan_workspace(s, select_mode, nsplit, workspace);
  if (w.total_bytes > workspace_bytes && w.cluster != nullptr && path != LOKI_PATH_CLUSTER)
    w = plan_workspace(s, select_mode, nsplit, workspace, false);  // no room for the exchange area: the other sequences
  if (w.total_bytes > workspace_bytes) return LOKI_ERR_WORKSPACE;

  hipStream_t st = static_cast<hipStream_t>(stream);
  const int heads_sel = (select_mode == 1) ? s.B * s.Hkv : s.B * s.Hq;
  int32_t* idx = out_idx ? out_idx : w.sel_idx;
  StageTimer tm(st);
  hipError_t e;
  if (path == LOKI_PATH_CLUSTER && (s.G == 1 || !fused_gqa_cluster_eligible(s, select_mode)))
    return LOKI_ERR_UNSUPPORTED;
  if (s.G == 1) {
    if (path == LOKI_PATH_FUSED && !fused_eligible(s)) return LOKI_ERR_UNSUPPORTED;
    if (path == LOKI_PATH_FUSED || (path == 0 && fused_preferred(s))) {
      tm.begin("fused_decode");
      e = launch_fused(s, q, P, klo, khi, v, out, out_idx, st);
      tm.end();
      return e == hipSuccess ? LOKI_OK : LOKI_ERR_HIP;
    }
  } else {
    if (path == LOKI_PATH_CLUSTER || (path == 0 && w.cluster != nullptr && fused_gqa_cluster_preferred(s, select_mode))) {
      tm.begin("fused_decode");
      e = launch_fused_gqa_cluster(s, q, P, klo, khi, v, out, out_idx, w.cluster_ctl, ws_zeroed, w.cluster, st);
      tm.end();
      return e == hipSuccess ? LOKI_OK : LOKI_ERR_HIP;
    }
    if (path == LOKI_PATH_FUSED && !fused_gqa_eligible(s, select_mode)) return LOKI_ERR_UNSUPPORTED;
    if (path == LOKI_PATH_FUSED || (path == 0 && fused_gqa_preferred(s, select_mode))) {
      tm.begin("fused_decode");
      e = launch_fused_gqa(s, q, P, klo, khi, v, out, out_idx, st);
      tm.end();
      return e == hipSuccess ? LOKI_OK : LOKI_ERR_HIP;
    }
  }
  // long sequences, one token each: the score kernel counts the leading key bits into the
  // chunk histograms at the head of the select scratch (cleared by the rotation kernel), and the
  // selection leaves its list as two ascending runs, merged only for the caller's copy
  const int hist_chunks = w.sel_scratch ? select_hist_chunks(s, select_mode) : 0;
  uint32_t* hist_part = hist_chunks ? w.sel_scratch : nullptr;
  if (hist_chunks) idx = w.sel_idx;
  tm.begin("rotate_query");
  // (the tickets lie directly before the select scratch, whose first words the histograms are)
  e = launch_qrot(s, q, P, w.qhat, klo, khi, v, reinterpret_cast<uint32_t*>(w.tickets),
                  w.ticket_words + (size_t)heads_sel * hist_chunks * 2048, st);
  tm.end();
  if (e != hipSuccess) return LOKI_ERR_HIP;
  tm.begin("score");
  e = launch_score(s, select_mode, q, P, klo, w.scores, w.qhat, hist_part, hist_chunks, st);
  tm.end();
  if (e != hipSuccess) return LOKI_ERR_HIP;
  tm.begin("select");
  e = launch_select(s, heads_sel, w.scores, idx, w.sel_score, w.sel_scratch, hist_chunks != 0,
                    hist_chunks ? out_idx : nullptr, st);
  tm.end();
  if (e != hipSuccess) return LOKI_ERR_HIP;
  tm.begin("gather_attend");
  // (with several row splits the block that finishes a head group last merges them)
  e = launch_gather(s, select_mode, nsplit, w.qhat, klo, khi, v, idx, w.sel_score, w.partial,
                    w.tickets, out, st);
  tm.end();
  return e == hipSuccess ? LOKI_OK : LOKI_ERR_HIP;
}

int loki_decode_attn(const loki_layout* layout, const void* q, const float* P, const void* klo,
                     const void* khi, const void* v, int S, int d, int k, int select_mode,
                     void* workspace, size_t workspace_bytes, void* out, int32_t* out_idx,
                     void* stream) {
  // nothing is appended, so the caches are only read
  return decode_impl(layout, q, P, const_cast<void*>(klo), const_cast<void*>(khi),
                     const_cast<void*>(v), S, d, k, select_mode, Ragged{}, Append{}, Paging{},
                     workspace, workspace_bytes, out, out_idx, stream);
}

int loki_decode_attn_static(const loki_layout* layout, const void* q, const float* P,
                            const void* klo, const void* khi, const void* v, int S, int d, int k,
                            int select_mode, void* out, int32_t* out_idx, void* stream) {
  size_t need = 0;
  const int rc = loki_workspace_bytes(layout, S, d, k, select_mode, &need);
  if (rc != LOKI_OK) return rc;
  if (need > (size_t)LOKI_STATIC_SCRATCH_BYTES) return LOKI_ERR_SCRATCH_LIMIT;
  void* ptr = nullptr;
  const int ra = static_scratch_address(&ptr);
  if (ra != LOKI_OK) return ra;
  // the array starts as zeros and only this library writes it: the condition of
  // LOKI_WORKSPACE_ZEROED (nothing else in the workspace has to start at zero)
  return decode_impl(layout, q, P, const_cast<void*>(klo), const_cast<void*>(khi),
                     const_cast<void*>(v), S, d, k, select_mode | LOKI_WORKSPACE_ZEROED, Ragged{}, Append{}, Paging{}, ptr,
                     (size_t)LOKI_STATIC_SCRATCH_BYTES, out, out_idx, stream);
}

int loki_decode_step(const loki_layout* layout, const void* q, const float* P, void* klo, void* khi,
                     void* v, int S_max, int d, int k_max, int select_mode,
                     const loki_step_args* args, void* workspace, size_t workspace_bytes, void* out,
                     int32_t* out_idx, void* stream) {
  Ragged rg;
  Append ap;
  Paging pg;
  if (args && args->page_table) {
    if (!layout) return LOKI_ERR_INVALID_ARG;
    const int rc = paging_from_args(args->page_table, args->page_rows, args->pages_per_seq,
                                    args->n_pages, layout->Hkv, S_max, &pg);
    if (rc != LOKI_OK) return rc;
  }
  if (args) {
    rg.seq_lens = args->seq_lens;
    rg.ks = args->ks;
    rg.queries = args->queries_per_seq > 0 ? args->queries_per_seq : 1;
    ap.k_new = args->k_new;
    ap.v_new = args->v_new;
  }
  return decode_impl(layout, q, P, klo, khi, v, S_max, d, k_max, select_mode, rg, ap, pg, workspace,
                     workspace_bytes, out, out_idx, stream);
}

static int dense_impl(const loki_layout* layout, const void* q, const void* k_full, const void* v,
                      int S, const int32_t* seq_lens, void* workspace, size_t workspace_bytes,
                      void* out, void* stream) {
  Shape s;
  loki_layout L;
  if (!layout) return LOKI_ERR_INVALID_ARG;
  L = *layout;
  L.d_split = 128;  // ignored by the dense path
  const int rc = check_layout(&L, &s);
  if (rc != LOKI_OK) return rc;
  if (!q || !k_full || !v || !out) return LOKI_ERR_INVALID_ARG;
  if (S < 1 || S > s.S_cap) return LOKI_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_full) || !aligned16(v) || !aligned16(out))
    return LOKI_ERR_ALIGNMENT;
  if (reinterpret_cast<uintptr_t>(seq_lens) & 3u) return LOKI_ERR_ALIGNMENT;
  s.S = S;
  s.rg.seq_lens = seq_lens;
  const int nsplit = dense_splits(s);
  const Workspace w = plan_workspace(s, -1, nsplit, workspace);
  if (nsplit > 1) {
    if (!workspace) return LOKI_ERR_INVALID_ARG;
    if (!aligned256(workspace)) return LOKI_ERR_ALIGNMENT;
    if (w.total_bytes > workspace_bytes) return LOKI_ERR_WORKSPACE;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  StageTimer tm(st);
  hipError_t e;
  tm.begin("dense_attend");
  e = launch_dense(s, nsplit, q, k_full, v, w.partial, out, st);
  tm.end();
  if (e != hipSuccess) return LOKI_ERR_HIP;
  if (nsplit > 1) {
    tm.begin("combine");
    e = launch_combine(s, nsplit, w.partial, out, st);
    tm.end();
    if (e != hipSuccess) return LOKI_ERR_HIP;
  }
  return LOKI_OK;
}

int dense_decode_attn(const loki_layout* layout, const void* q, const void* k_full, const void* v,
                      int S, void* workspace, size_t workspace_bytes, void* out, void* stream) {
  return dense_impl(layout, q, k_full, v, S, nullptr, workspace, workspace_bytes, out, stream);
}

int dense_decode_step(const loki_layout* layout, const void* q, const void* k_full, const void* v,
                      int S_max, const int32_t* seq_lens, void* workspace, size_t workspace_bytes,
                      void* out, void* stream) {
  return dense_impl(layout, q, k_full, v, S_max, seq_lens, workspace, workspace_bytes, out, stream);
}

int loki_pca_attn(const loki_layout* layout, const void* q, const float* P, const void* klo,
                  const void* v, int S, int d, void* workspace, size_t workspace_bytes, void* out,
                  void* stream) {
  Shape s;
  const int rc = check_layout(layout, &s);
  if (rc != LOKI_OK) return rc;
  if (!q || !P || !klo || !v || !out || !workspace) return LOKI_ERR_INVALID_ARG;
  if (S < 1 || S > s.S_cap) return LOKI_ERR_INVALID_ARG;
  if (d != s.d) return LOKI_ERR_UNSUPPORTED;
  if (!aligned16(q) || !aligned16(P) || !aligned16(klo) || !aligned16(v) || !aligned16(out))
    return LOKI_ERR_ALIGNMENT;
  if (!aligned256(workspace)) return LOKI_ERR_ALIGNMENT;
  s.S = S;
  const int nsplit = dense_splits(s);
  const Workspace w = plan_workspace(s, -2, nsplit, workspace);
  if (w.total_bytes > workspace_bytes) return LOKI_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  StageTimer tm(st);
  hipError_t e;
  tm.begin("rotate_query");
  e = launch_qrot(s, q, P, w.qhat, nullptr, nullptr, nullptr, nullptr, 0, st);
  tm.end();
  if (e != hipSuccess) return LOKI_ERR_HIP;
  tm.begin("pca_attend");
  e = launch_pca_attend(s, nsplit, w.qhat, klo, v, w.partial, out, st);
  tm.end();
  if (e != hipSuccess) return LOKI_ERR_HIP;
  if (nsplit > 1) {
    tm.begin("combine");
    e = launch_combine(s, nsplit, w.partial, out, st);
    tm.end();
    if (e != hipSuccess) return LOKI_ERR_HIP;
  }
  return LOKI_OK;
}

int loki_pca_workspace_bytes(const loki_layout* layout, long long n_rows, size_t* bytes) {
  Shape s;
  const int rc = check_layout(layout, &s);
  if (rc != LOKI_OK) return rc;
  if (!bytes || n_rows < 2 || n_rows > (1LL << 40)) return LOKI_ERR_INVALID_ARG;
  *bytes = pca_workspace_bytes(s.Hkv, n_rows);
  return LOKI_OK;
}

int loki_pca_fit(const loki_layout* layout, const void* keys, long long n_rows, float* P,
                 float* eigenvalues, void* workspace, size_t workspace_bytes, void* stream) {
  Shape s;
  const int rc = check_layout(layout, &s);
  if (rc != LOKI_OK) return rc;
  if (!keys || !P || !eigenvalues || !workspace) return LOKI_ERR_INVALID_ARG;
  if (n_rows < 2 || n_rows > (1LL << 40)) return LOKI_ERR_INVALID_ARG;
  if (!aligned16(keys) || !aligned16(P) || !aligned16(eigenvalues)) return LOKI_ERR_ALIGNMENT;
  if (!aligned256(workspace)) return LOKI_ERR_ALIGNMENT;
  if (pca_workspace_bytes(s.Hkv, n_rows) > workspace_bytes) return LOKI_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  StageTimer tm(st);
  static const char* const kStageNames[3] = {"pca_gram", "pca_covariance", "pca_eigensolve"};
  for (int stage = 0; stage < 3; ++stage) {
    tm.begin(kStageNames[stage]);
    const hipError_t e =
        launch_pca_stage(stage, s.Hkv, s.dtype, keys, n_rows, P, eigenvalues, workspace, st);
    tm.end();
    if (e != hipSuccess) return LOKI_ERR_HIP;
  }
  return LOKI_OK;
}

int loki_rank_at(const float* eigenvalues, int n_heads, int D, float v_percent, int32_t* ranks,
                 void* stream) {
  if (!eigenvalues || !ranks || n_heads < 1 || D < 1) return LOKI_ERR_INVALID_ARG;
  if (!(v_percent > 0.f) || v_percent > 100.f) return LOKI_ERR_INVALID_ARG;
  const hipError_t e = launch_rank_at(eigenvalues, n_heads, D, v_percent, ranks,
                                      static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LOKI_OK : LOKI_ERR_HIP;
}

int loki_layer_width(const float* eigenvalues, int n_heads, int D, float v_percent, int multiple,
                     float* mean_rank, int32_t* d_out, void* stream) {
  if (!eigenvalues || !d_out || n_heads < 1 || D < 1) return LOKI_ERR_INVALID_ARG;
  if (!(v_percent > 0.f) || v_percent > 100.f) return LOKI_ERR_INVALID_ARG;
  if (multiple < 1 || multiple > D || D % multiple != 0) return LOKI_ERR_INVALID_ARG;
  if ((long long)n_heads * D > 0x7fffffffLL / 2) return LOKI_ERR_UNSUPPORTED;  // rank sum in int32
  const hipError_t e = launch_layer_width(eigenvalues, n_heads, D, v_percent, multiple, mean_rank,
                                          d_out, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LOKI_OK : LOKI_ERR_HIP;
}

int loki_index_jaccard(const int32_t* idx_a, const int32_t* idx_b, int n_lists, int k, float* out,
                       void* stream) {
  if (!idx_a || !idx_b || !out || n_lists < 1 || k < 1) return LOKI_ERR_INVALID_ARG;
  const hipError_t e = launch_jaccard(idx_a, idx_b, n_lists, k, out, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LOKI_OK : LOKI_ERR_HIP;
}

int loki_profile_create(loki_profile** out) {
  if (!out) return LOKI_ERR_INVALID_ARG;
  loki_profile* p = new (std::nothrow) loki_profile();
  if (!p) return LOKI_ERR_INVALID_ARG;
  p->n = 0;
  for (int i = 0; i < 2 * LOKI_PROFILE_MAX_KERNELS; ++i) {
    if (hipEventCreate(&p->ev[i]) != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(p->ev[j]);
      delete p;
      return LOKI_ERR_HIP;
    }
  }
  *out = p;
  return LOKI_OK;
}

int loki_profile_destroy(loki_profile* p) {
  if (!p) return LOKI_ERR_INVALID_ARG;
  if (t_profile == p) t_profile = nullptr;
  for (int i = 0; i < 2 * LOKI_PROFILE_MAX_KERNELS; ++i) (void)hipEventDestroy(p->ev[i]);
  delete p;
  return LOKI_OK;
}

int loki_profile_attach(loki_profile* p) {
  t_profile = p;
  return LOKI_OK;
}

int loki_profile_read(loki_profile* p, int* n_kernels, float* ms, const char** names) {
  if (!p || !n_kernels || !ms) return LOKI_ERR_INVALID_ARG;
  *n_kernels = p->n;
  if (p->n == 0) return LOKI_OK;
  if (hipEventSynchronize(p->ev[2 * p->n - 1]) != hipSuccess) return LOKI_ERR_HIP;
  for (int i = 0; i < p->n; ++i) {
    if (hipEventElapsedTime(&ms[i], p->ev[2 * i], p->ev[2 * i + 1]) != hipSuccess)
      return LOKI_ERR_HIP;
    if (names) names[i] = p->names[i];
  }
  return LOKI_OK;
}

int loki_debug_cluster_spin_limit(unsigned polls) {
  set_cluster_spin_limit(polls ? polls : kClusterSpinLimit);
  return LOKI_OK;
}

int loki_cluster_gave_up(const void* workspace, int* gave_up, void* stream) {
  if (!workspace || !gave_up) return LOKI_ERR_INVALID_ARG;
  if (!aligned256(workspace)) return LOKI_ERR_ALIGNMENT;
  // the error word sits behind the control words of the last unit, at the start of the workspace
  const uint32_t* word = static_cast<const uint32_t*>(workspace) + (size_t)kClusterMaxUnits * kClusterCounterStride;
  uint32_t v = 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&v, word, sizeof(v), hipMemcpyDeviceToHost, st) != hipSuccess) return LOKI_ERR_HIP;
  if (hipStreamSynchronize(st) != hipSuccess) return LOKI_ERR_HIP;
  *gave_up = v != 0u ? 1 : 0;
  return LOKI_OK;
}

int loki_stream_read(const void* buf, size_t bytes, void* stream) {
  if (!buf || bytes == 0 || (bytes & 15) || (reinterpret_cast<uintptr_t>(buf) & 15))
    return LOKI_ERR_INVALID_ARG;
  hipLaunchKernelGGL(loki::stream_read_kernel, dim3(loki::device_cus()), dim3(512), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(buf), bytes / 16);
  return hipGetLastError() == hipSuccess ? LOKI_OK : LOKI_ERR_HIP;
}

}  // extern "C"
