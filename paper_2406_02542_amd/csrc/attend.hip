// Exact softmax attention over a list of cache rows (Algorithm 1 lines 7-9 of arXiv 2406.02542
// when the list is the selected set; Section 2 Eq. 1 when it is every row), with an online
// softmax in the log2 domain and scale 1/sqrt(D).
//
// One block owns a run of rows of one unit and NH query heads that share those rows.  A row
// of K (logical 128 columns, possibly split between the low-rank slab and the residual slab)
// and the matching row of V are each read by LPRV consecutive lanes with one 16-byte load per
// lane; the K.q dot product is finished with DPP inside the lane group; every lane keeps the
// running output for its EPC columns of V.  Partial (max, sum, output) triples are merged
// across lane groups, waves and finally across blocks (combine_kernel).
#include "attend_impl.h"

namespace loki {

constexpr int kAttThreads = 256;
constexpr int kAttWaves = kAttThreads / 64;

// LO_ONLY (with GATHER = false): every row, rotated query, logits from the low-rank slab alone
// (Appendix E, Algorithm 2).
template <typename T, int NH, bool GATHER, bool REUSE_LO, bool LO_ONLY = false>
__global__ __launch_bounds__(kAttThreads) void attend_kernel(
    const void* __restrict__ k_a,   // GATHER: klo [units, S_cap, d]; dense: K [units, S_cap, 128]
    const void* __restrict__ k_b,   // GATHER: khi [units, S_cap, 128-d]; dense: unused
    const void* __restrict__ v,     // [units, S_cap, 128]
    const void* __restrict__ qv,    // GATHER: qhat fp32 [B*Hq, 128]; dense: q storage [B*Hq, 128]
    const int32_t* __restrict__ sel_idx,   // GATHER: [blocks_y, n]
    const float* __restrict__ sel_score,   // REUSE_LO: [blocks_y, n] approximate scores of sel_idx
    float* partial,                 // [B*Hq, nsplit, 130] when nsplit > 1
    int32_t* tickets,               // [blocks_y] zeroed, or null: the merge of the splits is a launch of its own
    void* __restrict__ out,         // [B*Hq, 128] storage type; written here unless nsplit > 1 and no tickets
    int Hq, int Gq, int S_cap, int d, int n_max, int rows_per_block, int nsplit, int S_max, Ragged rag, Paging pg,
    int xcd_group_blocks, int xcd_sets) {
  using ST = typename T::store_t;
  constexpr int EPC = T::EPC;
  constexpr int LPRV = kD / EPC;           // lanes per row: 16 (bf16) or 32 (fp32)
  constexpr int RPW = 64 / LPRV;           // rows a wave covers per load instruction

  __shared__ int32_t s_idx[GATHER ? kMaxGatherChunk : 1];
  __shared__ float s_a[REUSE_LO ? kMaxGatherChunk : 1];
  __shared__ MergeSmem<kAttWaves, NH> s_merge;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane % LPRV, rg = lane / LPRV;
  // Which (split, head) this block is.  Blocks go to the 8 XCDs round-robin in launch order
  // and each XCD has its own L2.  Query heads that read the same KV head of the same sequence
  // (the G heads of a group when every head selects for itself, and the tokens of one
  // sequence when a step brings several) pick largely the same rows, so their blocks are
  // renumbered to land on one XCD, next to each other in time.  xcd_group_blocks = blocks of
  // one such set (0: launch order as is), xcd_sets = number of sets; the grid is rounded up to
  // a multiple of 8 sets and the blocks of the sets that do not exist leave at once.
  int bx = blockIdx.x, by = blockIdx.y;
  if (xcd_group_blocks > 0) {
    const int v = by * nsplit + bx;
    const int xcd = v & 7, j = v >> 3;
    const int set = (j / xcd_group_blocks) * 8 + xcd, m = j % xcd_group_blocks;
    if (set >= xcd_sets) return;  // uniform for the block, before any barrier
    const int member = m / nsplit;                 // (token, head of the group)
    const int Hkv = Hq / Gq, tokens = max(rag.queries, 1);
    const int seq = set / Hkv, hkv = set % Hkv;
    by = ((seq * tokens + member / Gq) * Hkv + hkv) * Gq + member % Gq;
    bx = m % nsplit;
  }
  const int head0 = by * NH;              // first query head, flattened over batch
  const int bidx = head0 / Hq;
  const int kv_unit = bidx * (Hq / Gq) + (head0 % Hq) / Gq;

  // list length of this sequence: the rows it keeps (gather: exactly what the select stage
  // computed) or the rows it holds (dense).  A block whose run starts past the end publishes
  // the neutral partial (max -big, sum 0).
  const int n = GATHER ? seq_keep(rag, bidx, n_max, seq_rows(rag, bidx, S_max))
                       : seq_rows(rag, bidx, n_max);
  const int r0 = bx * rows_per_block;
  const int r1 = min(n, r0 + rows_per_block);

  // a paged cache: the list in LDS holds rows of the pool and the slabs are addressed from their start
  const bool paged = GATHER && pg.table != nullptr;
  const int cache_b = bidx / max(rag.queries, 1);
  if constexpr (GATHER) {
    const int32_t* idx = sel_idx + (size_t)by * n_max;
    const int S_b = seq_rows(rag, bidx, S_max);
    for (int i = tid; i < r1 - r0; i += kAttThreads) {
      const int pos = min(max(idx[r0 + i], 0), S_b - 1);  // a bad list entry cannot leave the unit's rows
      s_idx[i] = paged ? (int32_t)cache_row(pg, cache_b, kv_unit % (Hq / Gq), Hq / Gq, S_cap, pos) : pos;
      if constexpr (REUSE_LO) s_a[i] = sel_score[(size_t)by * n_max + r0 + i];
    }
    __syncthreads();
  }

  // this lane's slice of the NH query vectors
  float qr[NH][EPC];
#pragma unroll
  for (int g = 0; g < NH; ++g) {
    if constexpr (GATHER || LO_ONLY) {
      const float* qh = static_cast<const float*>(qv) + (size_t)(head0 + g) * kD + c * EPC;
#pragma unroll
      for (int e = 0; e < EPC; ++e) qr[g][e] = qh[e];
    } else {
      const ST* qh = static_cast<const ST*>(qv) + (size_t)(head0 + g) * kD + c * EPC;
#pragma unroll
      for (int e = 0; e < EPC; ++e) qr[g][e] = T::load1(qh + e);
    }
  }

  const RowAddr ra = make_row_addr<T, REUSE_LO, LO_ONLY>(k_a, k_b, v,
                                                         paged ? (size_t)0 : (size_t)cache_unit(rag, kv_unit, Hq / Gq), S_cap,
                                                         (GATHER || LO_ONLY) ? d : kD, c);
  AttendAcc<T, NH> acc;
  acc.init();
  attend_rows<T, NH, kAttWaves * RPW, GATHER, REUSE_LO>(acc, qr, ra, s_idx, s_a, wave * RPW + rg,
                                                        r0, r1);
  attend_publish<T, NH, kAttWaves>(acc, s_merge);

  // thread t owns column t % 128 of heads t / 128, t / 128 + 2, ...
  for (int i = tid; i < NH * kD; i += kAttThreads) {
    const int g = i / kD, col = i % kD;
    float mn, ls, os;
    attend_merged<kAttWaves, NH>(s_merge, g, col, mn, ls, os);
    const size_t head = (size_t)(head0 + g);
    if (nsplit == 1) {
      T::store1(static_cast<ST*>(out) + head * kD + col, os / ls);
    } else {
      float* pr = partial + (head * nsplit + bx) * kPartialStride;
      const bool shared = tickets != nullptr;  // another block of this launch reads them
      store_shared_f32(pr + col, os, shared);
      if (col == 0) {
        store_shared_f32(pr + kD, mn, shared);
        store_shared_f32(pr + kD + 1, ls, shared);
      }
    }
  }
  if (nsplit > 1 && tickets != nullptr && splits_all_done(tickets + by, nsplit)) {
    for (int i = tid; i < NH * kD; i += kAttThreads) {
      const size_t head = (size_t)(head0 + i / kD);
      T::store1(static_cast<ST*>(out) + head * kD + i % kD,
                combine_splits<true>(partial + head * nsplit * kPartialStride, nsplit, i % kD));
    }
  }
}

// Merges the nsplit partial results of each query head (launches that have no ticket array:
// the dense baseline and Algorithm 2 of Appendix E).
template <typename T>
__global__ __launch_bounds__(kD) void combine_kernel(const float* __restrict__ partial,
                                                     typename T::store_t* __restrict__ out,
                                                     int nsplit) {
  const size_t head = blockIdx.x;
  const int col = threadIdx.x;
  T::store1(out + head * kD + col, combine_splits<false>(partial + head * nsplit * kPartialStride, nsplit, col));
}

// ---- launchers ------------------------------------------------------------------------
template <typename T, int NH, bool GATHER>
static hipError_t launch_attend_nh(int blocks_y, int nsplit, int rows_per_block, const void* k_a,
                                   const void* k_b, const void* v, const void* qv,
                                   const int32_t* sel_idx, const float* sel_score, float* partial,
                                   int32_t* tickets, void* out, int Hq, int Gq, int S_cap, int d, int n, int S_max,
                                   const Ragged& rg, const Paging& pg, int xcd_group_blocks,
                                   int xcd_sets, hipStream_t st) {
  // the saved ranking score replaces the low-rank slab read when one head owns the selection
  // (d = 128, Exact-TopK of Section 5: it is the whole logit and no key is read again)
  constexpr bool kCanReuse = GATHER && NH == 1;
  if (kCanReuse && sel_score != nullptr) {
    hipLaunchKernelGGL((attend_kernel<T, NH, GATHER, kCanReuse>), dim3(nsplit, blocks_y),
                       dim3(kAttThreads), 0, st, k_a, k_b, v, qv, sel_idx, sel_score, partial, tickets,
                       out, Hq, Gq, S_cap, d, n, rows_per_block, nsplit, S_max, rg, pg, xcd_group_blocks, xcd_sets);
  } else {
    hipLaunchKernelGGL((attend_kernel<T, NH, GATHER, false>), dim3(nsplit, blocks_y),
                       dim3(kAttThreads), 0, st, k_a, k_b, v, qv, sel_idx, sel_score, partial, tickets,
                       out, Hq, Gq, S_cap, d, n, rows_per_block, nsplit, S_max, rg, pg, xcd_group_blocks, xcd_sets);
  }
  return hipGetLastError();
}

template <typename T, bool GATHER>
static hipError_t launch_attend_t(int NH, int blocks_y, int nsplit, int rows_per_block,
                                  const void* k_a, const void* k_b, const void* v, const void* qv,
                                  const int32_t* sel_idx, const float* sel_score, float* partial,
                                  int32_t* tickets, void* out, int Hq, int Gq, int S_cap, int d, int n, int S_max,
                                  const Ragged& rg, const Paging& pg, int xcd_group_blocks,
                                  int xcd_sets, hipStream_t st) {
#define LOKI_ATT(NHV)                                                                          \
  return launch_attend_nh<T, NHV, GATHER>(blocks_y, nsplit, rows_per_block, k_a, k_b, v, qv,   \
                                          sel_idx, sel_score, partial, tickets, out, Hq, Gq, S_cap, d, n, S_max, rg, pg, \
                                          xcd_group_blocks, xcd_sets, st)
  switch (NH) {
    case 1: LOKI_ATT(1);
    case 2: LOKI_ATT(2);
    case 4: LOKI_ATT(4);
    case 8: LOKI_ATT(8);
    default: return hipErrorInvalidValue;
  }
#undef LOKI_ATT
}

static inline int div_up(int a, int b) { return (a + b - 1) / b; }

hipError_t launch_gather(const Shape& s, int select_mode, int nsplit, const float* qhat,
                         const void* klo, const void* khi, const void* v, const int32_t* sel_idx,
                         const float* sel_score, float* partial, int32_t* tickets, void* out,
                         hipStream_t st) {
  const int NH = (select_mode == 1) ? s.G : 1;
  if (attend_mfma_applies(s, NH))
    return launch_gather_mfma(s, nsplit, qhat, klo, khi, v, sel_idx, partial, tickets, out, st);
  int blocks_y = s.B * s.Hq / NH;
  const int rpb = div_up(s.k, nsplit);
  if (rpb > kMaxGatherChunk) return hipErrorInvalidValue;
  // query heads that read the same cached KV head share most rows: keep their blocks on one
  // XCD (see attend_kernel)
  const int tokens = s.rg.queries > 1 ? s.rg.queries : 1;
  const int sharers = tokens * s.G;
  const int sets = s.B / tokens * s.Hkv;
  int xcd = 0;
  if (NH == 1 && sharers > 1 && (long long)div_up(sets, 8) * 8 * sharers <= 65535) {
    xcd = sharers * nsplit;
    blocks_y = div_up(sets, 8) * 8 * sharers;
  }
  if (s.dtype == 0)
    return launch_attend_t<F32, true>(NH, blocks_y, nsplit, rpb, klo, khi, v, qhat, sel_idx,
                                      sel_score, partial, tickets, out, s.Hq, s.G, s.S_cap, s.d, s.k, s.S, s.rg, s.pg, xcd, sets, st);
  return launch_attend_t<BF16, true>(NH, blocks_y, nsplit, rpb, klo, khi, v, qhat, sel_idx,
                                     sel_score, partial, tickets, out, s.Hq, s.G, s.S_cap, s.d, s.k, s.S, s.rg, s.pg, xcd, sets, st);
}

hipError_t launch_dense(const Shape& s, int nsplit, const void* q, const void* k_full,
                        const void* v, float* partial, void* out, hipStream_t st) {
  if (attend_mfma_applies(s, s.G)) return launch_dense_mfma(s, nsplit, q, k_full, v, partial, out, st);
  const int blocks_y = s.B * s.Hkv;
  const int rpb = div_up(s.S, nsplit);
  if (s.dtype == 0)
    return launch_attend_t<F32, false>(s.G, blocks_y, nsplit, rpb, k_full, nullptr, v, q, nullptr,
                                       nullptr, partial, nullptr, out, s.Hq, s.G, s.S_cap, kD, s.S, s.S, s.rg, Paging{}, 0, 0, st);
  return launch_attend_t<BF16, false>(s.G, blocks_y, nsplit, rpb, k_full, nullptr, v, q, nullptr,
                                      nullptr, partial, nullptr, out, s.Hq, s.G, s.S_cap, kD, s.S, s.S, s.rg, Paging{}, 0, 0, st);
}

template <typename T, int NH>
static hipError_t launch_pca_nh(const Shape& s, int nsplit, int rpb, const float* qhat, const void* klo,
                                const void* v, float* partial, void* out, hipStream_t st) {
  hipLaunchKernelGGL((attend_kernel<T, NH, false, false, true>), dim3(nsplit, s.B * s.Hkv),
                     dim3(kAttThreads), 0, st, klo, nullptr, v, qhat, nullptr, nullptr, partial, nullptr,
                     out, s.Hq, s.G, s.S_cap, s.d, s.S, rpb, nsplit, s.S, s.rg, Paging{}, 0, 0);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_pca_t(const Shape& s, int nsplit, int rpb, const float* qhat, const void* klo,
                               const void* v, float* partial, void* out, hipStream_t st) {
  switch (s.G) {
    case 1: return launch_pca_nh<T, 1>(s, nsplit, rpb, qhat, klo, v, partial, out, st);
    case 2: return launch_pca_nh<T, 2>(s, nsplit, rpb, qhat, klo, v, partial, out, st);
    case 4: return launch_pca_nh<T, 4>(s, nsplit, rpb, qhat, klo, v, partial, out, st);
    case 8: return launch_pca_nh<T, 8>(s, nsplit, rpb, qhat, klo, v, partial, out, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_pca_attend(const Shape& s, int nsplit, const float* qhat, const void* klo,
                             const void* v, float* partial, void* out, hipStream_t st) {
  if (attend_mfma_applies(s, s.G)) return launch_pca_mfma(s, nsplit, qhat, klo, v, partial, out, st);
  const int rpb = div_up(s.S, nsplit);
  return s.dtype == 0 ? launch_pca_t<F32>(s, nsplit, rpb, qhat, klo, v, partial, out, st)
                      : launch_pca_t<BF16>(s, nsplit, rpb, qhat, klo, v, partial, out, st);
}

hipError_t launch_combine(const Shape& s, int nsplit, const float* partial, void* out,
                          hipStream_t st) {
  if (s.dtype == 0)
    hipLaunchKernelGGL(combine_kernel<F32>, dim3(s.B * s.Hq), dim3(kD), 0, st, partial,
                       static_cast<float*>(out), nsplit);
  else
    hipLaunchKernelGGL(combine_kernel<BF16>, dim3(s.B * s.Hq), dim3(kD), 0, st, partial,
                       static_cast<uint16_t*>(out), nsplit);
  return hipGetLastError();
}

}  // namespace loki
