// The whole decode step of Loki (Algorithm 1 lines 3 and 5-9 of arXiv 2406.02542) for one
// (batch, head) unit in ONE block, for shapes where a unit's scores fit in LDS and there are
// enough units to fill the chip: rotate q, score the low-rank slab into LDS, select the top-k
// in LDS, then attend over the selected rows — no score buffer, index list or partial result
// ever leaves the CU, and there is no launch boundary between the stages.
#include <type_traits>

#include "attend_impl.h"
#include "score_impl.h"
#include "select_impl.h"

namespace loki {

constexpr int kFusedThreads = 512;
constexpr int kFusedWaves = kFusedThreads / 64;
constexpr int kFusedKPT = kFusedMaxS / kFusedThreads;  // keys a thread may hold in the select stage

// positions per thread in the select stage: ceil(S / threads) rounded up to a multiple of 4
__host__ __device__ inline int fused_keys_per_thread(int S) {
  const int c = (S + kFusedThreads - 1) / kFusedThreads;
  return (c + 3) & ~3;
}

// Two blocks share a CU (4 waves per SIMD): the register budget is 128 VGPRs and the compiler
// is told not to trade load-level parallelism for a higher occupancy that cannot happen.
// KPT = keys a thread holds in the select stage (8 for S <= 4096, else 16).
// Which (sequence, head) unit a block works on.  Uniform batches: unit = block.  Ragged batches
// (up to 64 sequences): the sequences are ranked by length and handed out so that the two
// blocks that share a CU (block i and block i + half the grid, when the whole grid is resident)
// get a long and a short sequence: the first half of the grid takes the longest sequences in
// descending order, the second half the rest in ascending order.  Every wave computes the same
// answer from the length array (lane l ranks sequence l), so no barrier is needed.
__device__ __forceinline__ int fused_unit_of_block(const Ragged& rag, int B, int Hkv, int block) {
  if (rag.seq_lens == nullptr || B > 64 || B < 2) return block;
  const int lane = threadIdx.x & 63;
  const int mine = lane < B ? rag.seq_lens[lane] : 0;
  int rank = 0;
  for (int j = 0; j < B; ++j) {
    const int other = rag.seq_lens[j];
    rank += (other > mine || (other == mine && j < lane)) ? 1 : 0;
  }
  const int pos = block / Hkv, half = (B + 1) / 2;
  const int want = pos < half ? pos : B - 1 - (pos - half);
  const unsigned long long hit = __ballot(lane < B && rank == want);
  if (hit == 0ull) return block;              // cannot happen: the ranks are a permutation of 0..B-1
  const int b = __ffsll((long long)hit) - 1;  // exactly one lane holds each rank
  return b * Hkv + block % Hkv;
}

// APPEND: the block also rotates the unit's new key with the P_h entries it already holds and
// writes it, with the new value, into row S-1 of the unit's cache before it scores.  The block's
// own later reads of that row go through the same L1 and see it after the barrier; no other
// block reads this unit's rows.
constexpr int kFusedMaxPages = kFusedMaxS / 256;  // pages are at least 256 rows

// PAGED: the three slabs are pools addressed through the sequence's page list (see Paging).
template <typename T, int LPR, bool REUSE_LO, int KPT, bool APPEND, bool PAGED>
__global__ __launch_bounds__(kFusedThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void
fused_decode_kernel(
    const typename T::store_t* klo, const typename T::store_t* khi, const typename T::store_t* v,
    const typename T::store_t* __restrict__ q, const float* __restrict__ P,
    typename T::store_t* __restrict__ out, int32_t* __restrict__ out_idx, int Hkv, int S_max,
    int S_cap, int d, int k_max, Ragged rag, Append ap, Paging pg) {
  using ST = typename T::store_t;
  constexpr int EPC = T::EPC;
  constexpr int LPRV = kD / EPC;
  constexpr int RPW = 64 / LPRV;

  extern __shared__ __align__(16) unsigned char dyn_smem[];
  const int per_thread = fused_keys_per_thread(S_max);           // multiple of 4, <= kFusedKPT
  float* s_score = reinterpret_cast<float*>(dyn_smem);           // [kFusedThreads * per_thread]
  int32_t* s_idx = reinterpret_cast<int32_t*>(s_score + kFusedThreads * per_thread);  // [k_max]
  float* s_a = reinterpret_cast<float*>(s_idx + k_max);          // [k_max]

  __shared__ __align__(16) float s_q[kD];
  __shared__ __align__(8) float s_part[kRotParts][kD];
  __shared__ float s_qhat[1][kD];
  __shared__ __align__(16) float s_kn[APPEND ? kD : 4];                       // the new key
  __shared__ __align__(8) float s_partk[APPEND ? kRotParts : 1][APPEND ? kD : 2];
  static_assert(kFusedWaves == kRotParts, "one wave per part of the rotation");
  __shared__ ResidentSelectSmem<kFusedThreads> s_sel;
  __shared__ MergeSmem<kFusedWaves, 1> s_merge;
  __shared__ int32_t s_pages[PAGED ? kFusedMaxPages : 1];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // = b * H + h; one query head per KV head here
  const int unit = fused_unit_of_block(rag, (int)gridDim.x / Hkv, Hkv, (int)blockIdx.x);
  const int h = unit % Hkv;
  const int S = seq_rows(rag, unit / Hkv, S_max);
  const int k = seq_keep(rag, unit / Hkv, k_max, S);

  LOKI_STAMP(0);
#ifdef LOKI_PHASE_TIMING
  if (threadIdx.x == 0 && blockIdx.x < 8192) {
    g_phase_ts[blockIdx.x * kPhaseSlots + 9] = __builtin_amdgcn_s_getreg((31 << 11) | 4);    // HW_ID
    g_phase_ts[blockIdx.x * kPhaseSlots + 10] = __builtin_amdgcn_s_getreg((31 << 11) | 20);  // XCC_ID
  }
#endif
  resident_select_clear<kFusedThreads>(s_sel);  // covered by the barriers of the next stages

  // this lane's place in the low-rank slab
  const int cs = lane % LPR;
  const bool cact = cs < d / EPC;
  const size_t slab_row_bytes = (size_t)d * T::kBytes;
  using Rows = std::conditional_t<PAGED, PagedRows, ContiguousRows>;
  Rows slab;
  if constexpr (PAGED) {
    // the sequence's page list, clamped into the pool; readable after the first barrier below
    if (tid < kFusedMaxPages && tid < pg.pages_per_seq)
      s_pages[tid] = min(max(pg.table[(size_t)(unit / Hkv) * pg.pages_per_seq + tid], 0), pg.n_pages - 1);
    slab = PagedRows{reinterpret_cast<const char*>(klo) + (size_t)(cact ? cs : 0) * 16, slab_row_bytes,
                     s_pages, pg.lg_rows, Hkv, h};
  } else {
    slab = ContiguousRows{reinterpret_cast<const char*>(klo) + (size_t)unit * S_cap * slab_row_bytes +
                              (size_t)(cact ? cs : 0) * 16,
                          slab_row_bytes};
  }
  constexpr bool kPipelined = LPR <= 8;
  // Issue order = the order the results are needed in (loads return in order): q, then this
  // thread's 16 x 2 entries of P_h, then the first slab loads, which do not need qhat and stay
  // in flight during the rotation.
  const float q_mine = T::load1(q + (size_t)unit * kD + (tid & (kD - 1)));  // no branch: no early wait
  float kn_mine = 0.f, vn_mine = 0.f;
  if constexpr (APPEND) {
    kn_mine = T::load1(static_cast<const ST*>(ap.k_new) + (size_t)unit * kD + (tid & (kD - 1)));
    vn_mine = T::load1(static_cast<const ST*>(ap.v_new) + (size_t)unit * kD + (tid & (kD - 1)));
  }
  // qhat = q P_h with the association every path uses (8 parts of 16 terms, parts added in
  // order): wave w owns part w, lane l columns 2l and 2l+1; a load instruction of the wave
  // covers one 512-byte row of P_h.
  float2 pv[kRotPartLen];
  {
    const float* Ph = P + (size_t)h * kD * kD + (size_t)(wave * kRotPartLen) * kD + 2 * lane;
#pragma unroll
    for (int ii = 0; ii < kRotPartLen; ++ii)
      pv[ii] = *reinterpret_cast<const float2*>(Ph + (size_t)ii * kD);
  }
  ScoreTrip<kPipelined ? LPR : 8> first_trip, second_trip;
  constexpr int kTripRows = kFusedWaves * 64 * ScoreTrip<kPipelined ? LPR : 8>::TPI;
  if constexpr (kPipelined && !PAGED) {  // (a paged cache needs its page list in LDS first)
    score_load_trip<LPR, kFusedWaves>(slab, wave * 64, S, first_trip);
    if constexpr (!APPEND)  // the appending variant has no registers to spare during the rotation
      score_load_trip<LPR, kFusedWaves>(slab, wave * 64 + kTripRows, S, second_trip);
  }

  s_q[tid & (kD - 1)] = q_mine;  // four threads store the same value: no branch to sink the load into
  if constexpr (APPEND) s_kn[tid & (kD - 1)] = kn_mine;
  __syncthreads();
  if constexpr (kPipelined && PAGED && !APPEND) {  // the page list is in LDS now
    score_load_trip<LPR, kFusedWaves>(slab, wave * 64, S, first_trip);
    score_load_trip<LPR, kFusedWaves>(slab, wave * 64 + kTripRows, S, second_trip);
  }
  auto rotate_part = [&](const float* vec, float* part_row) {
    float a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int i4 = 0; i4 < kRotPartLen; i4 += 4) {
      const float4 qq = *reinterpret_cast<const float4*>(&vec[wave * kRotPartLen + i4]);
      a0 = fmaf(qq.x, pv[i4 + 0].x, a0);
      a1 = fmaf(qq.x, pv[i4 + 0].y, a1);
      a0 = fmaf(qq.y, pv[i4 + 1].x, a0);
      a1 = fmaf(qq.y, pv[i4 + 1].y, a1);
      a0 = fmaf(qq.z, pv[i4 + 2].x, a0);
      a1 = fmaf(qq.z, pv[i4 + 2].y, a1);
      a0 = fmaf(qq.w, pv[i4 + 3].x, a0);
      a1 = fmaf(qq.w, pv[i4 + 3].y, a1);
    }
    *reinterpret_cast<float2*>(&part_row[2 * lane]) = make_float2(a0, a1);
  };
  rotate_part(s_q, s_part[wave]);
  if constexpr (APPEND) rotate_part(s_kn, s_partk[wave]);
  __syncthreads();
  if (tid < kD) {
    float sum = 0.f;
#pragma unroll
    for (int pp = 0; pp < kRotParts; ++pp) sum += s_part[pp][tid];
    s_qhat[0][tid] = sum;
  }
  if constexpr (APPEND) {
    // row S-1 of the unit's cache: rotated key (columns < d to the low-rank slab, the rest to
    // the residual slab) by threads 128..255, value by threads 256..383
    size_t row;
    if constexpr (PAGED) row = (size_t)slab.pool_row(S - 1);
    else row = (size_t)unit * S_cap + (size_t)(S - 1);
    if (tid >= kD && tid < 2 * kD) {
      const int j = tid - kD;
      float sum = 0.f;
#pragma unroll
      for (int pp = 0; pp < kRotParts; ++pp) sum += s_partk[pp][j];
      ST* dst = j < d ? const_cast<ST*>(klo) + row * d + j : const_cast<ST*>(khi) + row * (kD - d) + (j - d);
      T::store1(dst, sum);
    } else if (tid >= 2 * kD && tid < 3 * kD) {
      T::store1(const_cast<ST*>(v) + row * kD + (tid - 2 * kD), vn_mine);
    }
  }
  __syncthreads();
  if constexpr (APPEND && kPipelined) {
    // the loads put in flight before the rotation may have read row S-1 before it was written
    if (PAGED || S - 1 < kTripRows)
      score_load_trip<LPR, kFusedWaves>(slab, wave * 64, S, first_trip);
    score_load_trip<LPR, kFusedWaves>(slab, wave * 64 + kTripRows, S, second_trip);
  }

  LOKI_STAMP(1);
  // ---- approximate scores over the low-rank slab, into LDS ------------------------------
  {
    float qr[1][EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) qr[0][e] = cact ? s_qhat[0][cs * EPC + e] : 0.f;
    auto to_lds = [&](int row, const float (&sc)[1]) { s_score[row] = sc[0]; };
    if constexpr (kPipelined)
      score_rows_pipelined<T, LPR, 1, kFusedWaves>(slab, qr, 0, S, first_trip, second_trip, to_lds);
    else
      score_rows<T, LPR, 1, kFusedWaves>(slab, cact, qr, 0, S, to_lds);
  }
  __syncthreads();
  LOKI_STAMP(2);

  // ---- top-k in LDS ------------------------------------------------------------------------
  int32_t* gidx = out_idx ? out_idx + (size_t)unit * k_max : nullptr;
  if (gidx)
    for (int i = k + tid; i < k_max; i += kFusedThreads) gidx[i] = -1;  // a sequence keeping fewer rows
  block_select_topk_resident<kFusedThreads, KPT>(s_score, S, k, per_thread, s_sel,
                                                       [&](int rank, int pos, float score) {
    if constexpr (PAGED) s_idx[rank] = (int32_t)slab.pool_row(pos);  // the attention stage reads pool rows
    else s_idx[rank] = pos;
    s_a[rank] = score;
    if (gidx) gidx[rank] = pos;
  });
  __syncthreads();
  LOKI_STAMP(6);

  // ---- exact attention over the selected rows -----------------------------------------------
  const int c = lane % LPRV, rg = lane / LPRV;
  float qr[1][EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) qr[0][e] = s_qhat[0][c * EPC + e];
  const RowAddr ra = make_row_addr<T, REUSE_LO>(klo, khi, v, PAGED ? (size_t)0 : (size_t)unit, S_cap, d, c);
  AttendAcc<T, 1> acc;
  acc.init();
  attend_rows<T, 1, kFusedWaves * RPW, true, REUSE_LO>(acc, qr, ra, s_idx, s_a, wave * RPW + rg, 0,
                                                       k);
  LOKI_STAMP(7);
  attend_publish<T, 1, kFusedWaves>(acc, s_merge);
  if (tid < kD) {
    float mn, ls, os;
    attend_merged<kFusedWaves, 1>(s_merge, 0, tid, mn, ls, os);
    T::store1(out + (size_t)unit * kD + tid, os / ls);
  }
  LOKI_STAMP(8);
}

#ifdef LOKI_PHASE_TIMING
extern "C" int loki_debug_read_phase_ts(unsigned long long* host_dst, size_t count) {
  return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(loki::g_phase_ts), count * sizeof(unsigned long long));
}
#endif

size_t fused_dynamic_lds(const Shape& s) {
  return (size_t)kFusedThreads * fused_keys_per_thread(s.S) * 4 + (size_t)s.k * 8;
}

bool fused_eligible(const Shape& s) {
  // several new tokens per sequence: a block would read rows appended by other blocks of the launch
  if (s.rg.queries > 1) return false;
  if (s.pg.table != nullptr && s.pg.pages_per_seq > kFusedMaxS / 256) return false;  // page list in LDS
  return s.G == 1 && s.S <= kFusedMaxS && s.k <= kFusedMaxK;
}

bool fused_preferred(const Shape& s) {
  if (!fused_eligible(s)) return false;
  const int units = s.B * s.Hkv;
  // measured on the Llama-2-shaped layer (S = 4096 and 8192): equal at 32 units, the single
  // launch ahead from 64 units on (25 vs 27 us) and by a third at 128 and more; below that only
  // when there is so little work per unit that the launch count dominates
  return units >= 48 || s.S <= 2048;
}

template <typename T, int LPR, bool REUSE_LO, int KPT, bool APPEND, bool PAGED>
static hipError_t launch_fused_k(const Shape& s, const void* q, const float* P, void* klo, void* khi,
                                 void* v, void* out, int32_t* out_idx, hipStream_t st) {
  using ST = typename T::store_t;
  auto kern = fused_decode_kernel<T, LPR, REUSE_LO, KPT, APPEND, PAGED>;
  const size_t lds = fused_dynamic_lds(s);
  static std::atomic<unsigned long long> lds_allowed{0};  // per instantiation: devices already set up
  const hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void*>(kern),
                                          (int)(kFusedMaxS * 4 + kFusedMaxK * 8), lds_allowed);
  if (ea != hipSuccess) return ea;
  hipLaunchKernelGGL(kern, dim3(s.B * s.Hkv), dim3(kFusedThreads), lds, st,
                     static_cast<const ST*>(klo), static_cast<const ST*>(khi),
                     static_cast<const ST*>(v), static_cast<const ST*>(q), P, static_cast<ST*>(out),
                     out_idx, s.Hkv, s.S, s.S_cap, s.d, s.k, s.rg, s.ap, s.pg);
  return hipGetLastError();
}

template <typename T, int LPR, bool REUSE_LO, int KPT>
static hipError_t launch_fused_a(const Shape& s, const void* q, const float* P, void* klo, void* khi,
                                 void* v, void* out, int32_t* out_idx, hipStream_t st) {
  const bool paged = s.pg.table != nullptr;
  if (s.ap.k_new != nullptr) {
    if (paged) return launch_fused_k<T, LPR, REUSE_LO, KPT, true, true>(s, q, P, klo, khi, v, out, out_idx, st);
    return launch_fused_k<T, LPR, REUSE_LO, KPT, true, false>(s, q, P, klo, khi, v, out, out_idx, st);
  }
  if (paged) return launch_fused_k<T, LPR, REUSE_LO, KPT, false, true>(s, q, P, klo, khi, v, out, out_idx, st);
  return launch_fused_k<T, LPR, REUSE_LO, KPT, false, false>(s, q, P, klo, khi, v, out, out_idx, st);
}

template <typename T, int LPR, bool REUSE_LO>
static hipError_t launch_fused_r(const Shape& s, const void* q, const float* P, void* klo, void* khi,
                                 void* v, void* out, int32_t* out_idx, hipStream_t st) {
  if (fused_keys_per_thread(s.S) <= 8)
    return launch_fused_a<T, LPR, REUSE_LO, 8>(s, q, P, klo, khi, v, out, out_idx, st);
  return launch_fused_a<T, LPR, REUSE_LO, kFusedKPT>(s, q, P, klo, khi, v, out, out_idx, st);
}

template <typename T, int LPR>
static hipError_t launch_fused_l(const Shape& s, const void* q, const float* P, void* klo, void* khi,
                                 void* v, void* out, int32_t* out_idx, hipStream_t st) {
  // the ranking score is reused as the low-rank part of the exact logit; with d = 128
  // (Exact-TopK of Section 5) it is the whole logit and the attention stage reads no key
  return launch_fused_r<T, LPR, true>(s, q, P, klo, khi, v, out, out_idx, st);
}

template <typename T>
static hipError_t launch_fused_t(const Shape& s, const void* q, const float* P, void* klo, void* khi,
                                 void* v, void* out, int32_t* out_idx, hipStream_t st) {
  const int nch = s.d / T::EPC;
  int lpr = 1;
  while (lpr < nch) lpr <<= 1;
  switch (lpr) {
    case 1: return launch_fused_l<T, 1>(s, q, P, klo, khi, v, out, out_idx, st);
    case 2: return launch_fused_l<T, 2>(s, q, P, klo, khi, v, out, out_idx, st);
    case 4: return launch_fused_l<T, 4>(s, q, P, klo, khi, v, out, out_idx, st);
    case 8: return launch_fused_l<T, 8>(s, q, P, klo, khi, v, out, out_idx, st);
    case 16: return launch_fused_l<T, 16>(s, q, P, klo, khi, v, out, out_idx, st);
    case 32:
      if constexpr (T::EPC == 4) return launch_fused_l<T, 32>(s, q, P, klo, khi, v, out, out_idx, st);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_fused(const Shape& s, const void* q, const float* P, void* klo, void* khi,
                        void* v, void* out, int32_t* out_idx, hipStream_t st) {
  if (!fused_eligible(s)) return hipErrorInvalidValue;
  return s.dtype == 0 ? launch_fused_t<F32>(s, q, P, klo, khi, v, out, out_idx, st)
                      : launch_fused_t<BF16>(s, q, P, klo, khi, v, out, out_idx, st);
}

}  // namespace loki
