// Attention over a list of cache rows for SEVERAL query heads that share those rows (grouped
// queries; Section 2 Eq. 1 for the dense baseline, Algorithm 1 lines 7-9 of arXiv 2406.02542
// for a selection shared by a KV group), bf16 caches, on the matrix cores.
//
// With NH heads per row both products are small dense contractions, and on the vector units
// their cost (NH x 128 multiply-adds per row, twice, plus NH softmax scalars evaluated by every
// lane of a row) outweighs the HBM time from about 8 heads on.  Here a wave works on steps of
// 32 rows:
//   S[row, head] = K[row, :] . q[head, :]      v_mfma_f32_16x16x32_bf16, A = the 16-byte-per-lane
//                                              load of a 16-row tile of K, B = q^T (16 heads)
//   softmax scalars per head                   lane (head, k-group) sees 8 of the 32 rows; the
//                                              step maximum is shared with two cross-row moves
//   O[head, col] += P[head, row] V[row, col]   A = P straight from the accumulator layout of the
//                                              first product (two bf16 terms), B = V^T, which
//                                              needs rows contiguous per lane: V tiles pass
//                                              through LDS (row pitch 264 B, conflict-free
//                                              2-byte column reads)
// q is bf16 for the dense baseline (exact).  The rotated query of the gather is fp32 and enters
// as two bf16 terms (16 significant bits): unlike the ranking scores, these logits decide no
// index, and a relative error of 2^-17 in them is far below the bf16 rounding of the output;
// the third term would cost 16 registers and a third of the first product's matrix work.
// The tile loop (attend_mfma_impl.h) keeps the next step's loads in flight during the softmax
// and the second product, which costs registers: two blocks share a CU.
#include "attend_mfma_impl.h"

namespace loki {

constexpr int kAmThreads = 256;
constexpr int kAmWaves = kAmThreads / 64;

// QT = number of bf16 terms q enters with (1: q is bf16; 2: q is fp32)
// KSTEPS / LO_ONLY (with GATHER = false): the logits use only the first d columns, held by k_a
// with row pitch d (Appendix E, Algorithm 2): KSTEPS = ceil(d / 32) of the four 32-column
// steps of the first product are issued, and columns past d (a partial last step) meet a zero
// in the B operand, so whatever valid chunk their lanes load does not count.
template <int NH, bool GATHER, int KSTEPS = 4, bool LO_ONLY = false>
__global__ __launch_bounds__(kAmThreads, 2) void attend_mfma_kernel(
    const void* __restrict__ k_a,   // GATHER: klo [units, S_cap, d]; dense: K [units, S_cap, 128]
    const void* __restrict__ k_b,   // GATHER: khi [units, S_cap, 128-d]; dense: unused
    const void* __restrict__ v,     // [units, S_cap, 128]
    const void* __restrict__ qv,    // GATHER: qhat fp32 [B*Hq, 128]; dense: q bf16 [B*Hq, 128]
    const int32_t* __restrict__ sel_idx,  // GATHER: [blocks_y, n]
    float* partial,                 // [B*Hq, nsplit, 130] when nsplit > 1
    int32_t* tickets,               // [KV units] zeroed, or null: the merge of the splits is a launch of its own
    uint16_t* __restrict__ out,     // [B*Hq, 128] bf16; written here unless nsplit > 1 and no tickets
    int S_cap, int d, int n_max, int rows_per_block, int nsplit, int Hkv, int S_max, Ragged rg,
    Paging pg) {
  constexpr bool kRotated = GATHER || LO_ONLY;  // the query is the fp32 rotated one
  constexpr int QT = kRotated ? 2 : 1;
  __shared__ __align__(16) unsigned char s_v[kAmWaves][kAmStageBytes];  // 8448 B per wave
  __shared__ int32_t s_idx[GATHER ? kMaxGatherChunk : 1];
  __shared__ MergeSmem<kAmWaves, NH> s_merge;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, kgrp = lane >> 4;
  const int kv_unit = blockIdx.y;          // one block row per KV unit: its NH heads share the rows
  const size_t head0 = (size_t)kv_unit * NH;
  const bool head_ok = r16 < NH;

  // list length of this sequence: the rows it keeps (gather) or holds (dense); a block whose
  // run starts past the end publishes the neutral partial
  const int bidx = kv_unit / Hkv;
  const int n = GATHER ? seq_keep(rg, bidx, n_max, seq_rows(rg, bidx, S_max))
                       : seq_rows(rg, bidx, n_max);
  const int r0 = blockIdx.x * rows_per_block;
  const int r1 = min(n, r0 + rows_per_block);

  // a paged cache: the list in LDS holds rows of the pool and the slabs are addressed from their start
  const bool paged = GATHER && pg.table != nullptr;
  if constexpr (GATHER) {
    const int32_t* idx = sel_idx + (size_t)blockIdx.y * n_max;
    const int cache_b = bidx / max(rg.queries, 1);
    const int S_b = seq_rows(rg, bidx, S_max);
    for (int i = tid; i < r1 - r0; i += kAmThreads) {
      const int pos = min(max(idx[r0 + i], 0), S_b - 1);  // a bad list entry cannot leave the unit's rows
      s_idx[i] = paged ? (int32_t)cache_row(pg, cache_b, kv_unit % Hkv, Hkv, S_cap, pos) : pos;
    }
    __syncthreads();
  }
  const size_t addr_unit = paged ? (size_t)0 : (size_t)cache_unit(rg, kv_unit, Hkv);

  // B operand of the first product: q of head r16, columns 32*step + 8*kgrp .. +7
  am_bf16x8_t bq[KSTEPS][QT];
  if constexpr (kRotated) {
    am_query_operands<KSTEPS, QT>(static_cast<const float*>(qv) + (head0 + (head_ok ? r16 : 0)) * kD,
                                  head_ok, LO_ONLY ? d : kD, bq);
  } else {
#pragma unroll
    for (int step = 0; step < KSTEPS; ++step) {
      const int col = 32 * step + 8 * kgrp;
      const uint16_t* qh = static_cast<const uint16_t*>(qv) + (head0 + (head_ok ? r16 : 0)) * kD + col;
      uint4 raw = load16(qh);
      if (!head_ok) raw = make_uint4(0, 0, 0, 0);
      bq[step][0] = __builtin_bit_cast(am_bf16x8_t, raw);
    }
  }

  const AmAddr<KSTEPS> ad = am_make_addr<KSTEPS, LO_ONLY>(k_a, k_b, v, addr_unit, S_cap, kRotated ? d : kD);
  AmState st;
  st.init();
  am_attend_rows<GATHER, KSTEPS, QT, kAmWaves>(ad, bq, s_idx, r0, r1, s_v[wave], st);
  am_publish<NH, kAmWaves>(st, s_merge);

  for (int i = tid; i < NH * kD; i += kAmThreads) {
    const int g = i / kD, col = i % kD;
    float mn, ls, os;
    attend_merged<kAmWaves, NH>(s_merge, g, col, mn, ls, os);
    const size_t head = head0 + g;
    if (nsplit == 1) {
      out[head * kD + col] = BF16::round(os / ls);
    } else {
      float* pr = partial + (head * nsplit + blockIdx.x) * kPartialStride;
      const bool shared = tickets != nullptr;  // another block of this launch reads them
      store_shared_f32(pr + col, os, shared);
      if (col == 0) {
        store_shared_f32(pr + kD, mn, shared);
        store_shared_f32(pr + kD + 1, ls, shared);
      }
    }
  }
  if (nsplit > 1 && tickets != nullptr && splits_all_done(tickets + kv_unit, nsplit)) {
    for (int i = tid; i < NH * kD; i += kAmThreads) {
      const size_t head = head0 + i / kD;
      out[head * kD + i % kD] =
          BF16::round(combine_splits<true>(partial + head * nsplit * kPartialStride, nsplit, i % kD));
    }
  }
}

template <bool GATHER>
static hipError_t launch_attend_mfma_nh(int NH, int blocks_y, int nsplit, int rpb, const void* k_a,
                                        const void* k_b, const void* v, const void* qv,
                                        const int32_t* sel_idx, float* partial, int32_t* tickets,
                                        void* out, int S_cap, int d, int n, int Hkv, int S_max, const Ragged& rg,
                                        const Paging& pg, hipStream_t st) {
  const dim3 grid(nsplit, blocks_y), block(kAmThreads);
  uint16_t* o16 = static_cast<uint16_t*>(out);
  switch (NH) {
    case 4:
      hipLaunchKernelGGL((attend_mfma_kernel<4, GATHER>), grid, block, 0, st, k_a, k_b, v, qv, sel_idx,
                         partial, tickets, o16, S_cap, d, n, rpb, nsplit, Hkv, S_max, rg, pg);
      break;
    case 8:
      hipLaunchKernelGGL((attend_mfma_kernel<8, GATHER>), grid, block, 0, st, k_a, k_b, v, qv, sel_idx,
                         partial, tickets, o16, S_cap, d, n, rpb, nsplit, Hkv, S_max, rg, pg);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int NH>
static hipError_t launch_pca_mfma_nh(const Shape& s, int nsplit, int rpb, const float* qhat,
                                     const void* klo, const void* v, float* partial, void* out,
                                     hipStream_t st) {
  const dim3 grid(nsplit, s.B * s.Hkv), block(kAmThreads);
  uint16_t* o16 = static_cast<uint16_t*>(out);
#define LOKI_PCA_MFMA(KS)                                                                          \
  hipLaunchKernelGGL((attend_mfma_kernel<NH, false, KS, true>), grid, block, 0, st, klo, nullptr, v, \
                     qhat, nullptr, partial, nullptr, o16, s.S_cap, s.d, s.S, rpb, nsplit, s.Hkv, s.S, s.rg,  \
                     Paging{});                                                                    \
  break
  switch ((s.d + 31) / 32) {
    case 1: LOKI_PCA_MFMA(1);
    case 2: LOKI_PCA_MFMA(2);
    case 3: LOKI_PCA_MFMA(3);
    case 4: LOKI_PCA_MFMA(4);
    default: return hipErrorInvalidValue;
  }
#undef LOKI_PCA_MFMA
  return hipGetLastError();
}

hipError_t launch_pca_mfma(const Shape& s, int nsplit, const float* qhat, const void* klo,
                           const void* v, float* partial, void* out, hipStream_t st) {
  const int rpb = (s.S + nsplit - 1) / nsplit;
  if (s.G == 8) return launch_pca_mfma_nh<8>(s, nsplit, rpb, qhat, klo, v, partial, out, st);
  if (s.G == 4) return launch_pca_mfma_nh<4>(s, nsplit, rpb, qhat, klo, v, partial, out, st);
  return hipErrorInvalidValue;
}

bool attend_mfma_applies(const Shape& s, int heads_per_block) {
  return s.dtype == 1 && (heads_per_block == 8 || heads_per_block == 4);
}

hipError_t launch_dense_mfma(const Shape& s, int nsplit, const void* q, const void* k_full,
                             const void* v, float* partial, void* out, hipStream_t st) {
  const int rpb = (s.S + nsplit - 1) / nsplit;
  return launch_attend_mfma_nh<false>(s.G, s.B * s.Hkv, nsplit, rpb, k_full, nullptr, v, q, nullptr,
                                      partial, nullptr, out, s.S_cap, kD, s.S, s.Hkv, s.S, s.rg, Paging{}, st);
}

hipError_t launch_gather_mfma(const Shape& s, int nsplit, const float* qhat, const void* klo,
                              const void* khi, const void* v, const int32_t* sel_idx, float* partial,
                              int32_t* tickets, void* out, hipStream_t st) {
  const int rpb = (s.k + nsplit - 1) / nsplit;
  if (rpb > kMaxGatherChunk) return hipErrorInvalidValue;
  return launch_attend_mfma_nh<true>(s.G, s.B * s.Hkv, nsplit, rpb, klo, khi, v, qhat, sel_idx,
                                     partial, tickets, out, s.S_cap, s.d, s.k, s.Hkv, s.S, s.rg, s.pg, st);
}

}  // namespace loki
