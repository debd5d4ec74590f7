// The single-launch decode step for grouped query heads (see fused_gqa.hip): the kernel itself,
// shared by the one-block-per-unit launch (fused_gqa.hip) and the launch that puts several
// cooperating blocks on a unit (fused_gqa_cluster.hip).
#pragma once

#include "attend_mfma_impl.h"
#include "cluster_impl.h"
#include "score_impl.h"
#include "score_mfma_impl.h"
#include "select_impl.h"

namespace loki {

constexpr int kGqaMaxK = kMaxGatherChunk;  // the index list lives in LDS
constexpr int kGqaMaxPages = 64;           // a paged cache: 16384 rows in pages of at least 256
// 16-byte slab loads a lane keeps in flight in the scoring stage (measured on the 64/8-head
// shapes at S = 8192: 64-byte slab rows gain 6 % from 16 against 8, the other widths nothing)
#ifndef LOKI_GQA_SCORE_DEPTH
#define LOKI_GQA_SCORE_DEPTH(NCH) ((NCH) == 4 ? 16 : 8)
#endif

// positions per thread in the select stage: ceil(S / threads) rounded up to a power of two (>= 4)
__host__ __device__ inline int gqa_keys_per_thread(int S, int threads) {
  const int c = (S + threads - 1) / threads;
  int p = 4;
  while (p < c) p *= 2;
  return p;
}

// LDS of one block beyond the static part: one region that the stages use in turn — the
// rotation's partial sums; then the score keys (padded, select_impl.h) followed by the list of
// threshold-bin candidates; then the value tiles of the attention stage; then the merge of the
// waves — and behind it the index list.
// CLUSTER (several blocks per unit, each on a slice of the rows): S is the longest slice, k
// the longest list a block can end up with; the candidates' keys live in device memory, only
// their positions in LDS.
template <int THREADS, int G, bool CLUSTER = false>
struct GqaLds {
  static constexpr int kWaves = THREADS / 64;
  static constexpr size_t kRotBytes = (size_t)(G + 1) * (kRotParts + 1) * kD * sizeof(float);  // partial sums + vectors (G queries, the new key)
  static constexpr size_t kStageBytes = (size_t)kWaves * kAmStageBytes;
  static constexpr size_t kMergeBytes = sizeof(MergeSmem<kWaves, G>);
  static constexpr int kCandPerThread = 8;
  static constexpr int kCandCap = kCandPerThread * THREADS;  // threshold-bin candidates kept as a compact list
  static constexpr size_t kCandBytes = (size_t)kCandCap * (CLUSTER ? 4 : 8);  // (key, position)
  __host__ __device__ static size_t cand_offset(int S) {
    const size_t b = padded_words((size_t)THREADS * gqa_keys_per_thread(S, THREADS)) * sizeof(uint32_t);
    return (b + 15) & ~(size_t)15;
  }
  __host__ __device__ static size_t region_bytes(int S) {
    size_t b = cand_offset(S) + kCandBytes;
    b = b > kRotBytes ? b : kRotBytes;
    b = b > kStageBytes ? b : kStageBytes;
    b = b > kMergeBytes ? b : kMergeBytes;
    return (b + 15) & ~(size_t)15;
  }
  __host__ __device__ static size_t total_bytes(int S, int k) { return region_bytes(S) + (size_t)k * 4; }
};

// Rows of a slice when C blocks share a unit of S rows: equal parts in whole 64-row groups.
__host__ __device__ inline int gqa_slice_rows(int S, int C) { return ((S + C - 1) / C + 63) / 64 * 64; }

// THREADS = 256: two blocks share a CU (S <= 8192); 512: one block per CU (S <= 16384).
// NCH = 16-byte chunks per slab row (d = 8 NCH); KPT = keys a thread holds in the select stage.
// PAGED: the three slabs are pools addressed through the sequence's page list (see Paging): the
// list sits in LDS, every slab load looks its page up, and the selected positions are translated
// to pool rows before the attention stage.
// CLUSTER: cl.C blocks work on one unit, block c on rows [c L, (c + 1) L) of it (L =
// gqa_slice_rows); they find the threshold together (cluster_impl.h), each attends over the
// selected rows of its slice, and the block that finishes last merges the partial results.
template <int THREADS, int NCH, int G, int KPT, bool PAGED, bool CLUSTER = false>
__global__ __launch_bounds__(THREADS, THREADS == 256 ? 2 : 1) void fused_gqa_kernel(
    const uint16_t* klo, const uint16_t* khi, const uint16_t* v,
    const uint16_t* __restrict__ q, const float* __restrict__ P, uint16_t* __restrict__ out,
    int32_t* __restrict__ out_idx, int Hkv, int S_max, int S_cap, int k_max, Ragged rag, Append ap,
    Paging pg, ClusterArgs cl) {
  constexpr int kWaves = THREADS / 64;
  constexpr int PPW = kRotParts / kWaves;  // parts of the rotation a wave owns
  static_assert(PPW * kWaves == kRotParts, "the rotation's 8 parts divide over the waves");
  constexpr int d = 8 * NCH;
  using Lds = GqaLds<THREADS, G, CLUSTER>;

  extern __shared__ __align__(16) unsigned char dyn_smem[];
  uint32_t* s_key = reinterpret_cast<uint32_t*>(dyn_smem);                 // scoring, select: keys of the scores
  float* s_q = reinterpret_cast<float*>(dyn_smem);                          // rotation: [G + 1][128]
  float* s_part = s_q + (G + 1) * kD;                                       // rotation: [G + 1][8][128]
  unsigned char* s_stage = dyn_smem;                                        // attention: value tiles
  MergeSmem<kWaves, G>& s_merge = *reinterpret_cast<MergeSmem<kWaves, G>*>(dyn_smem);  // merge
  // rows of the longest slice (CLUSTER) / of the longest sequence: what the score region is laid out for
  const int L_max = CLUSTER ? gqa_slice_rows(S_max, cl.C) : S_max;
  int32_t* s_idx = reinterpret_cast<int32_t*>(dyn_smem + Lds::region_bytes(L_max));  // [min(k_max, L_max)]
  __shared__ __align__(16) float s_qhat[G][kD];
  __shared__ int32_t s_pages[PAGED ? kGqaMaxPages : 1];
  __shared__ ResidentSelectSmem<THREADS> s_sel;
  __shared__ ClusterSmem s_cl;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15;
  // CLUSTER: workgroup ids are dealt to the 8 XCDs in turn; the members of a unit are ids 8 apart
  // (the same XCD, dispatched one after the other), and a launch is padded to whole rows of 8 units
  const int unit = CLUSTER ? (int)(blockIdx.x / 8 / cl.C) * 8 + (int)(blockIdx.x % 8) : (int)blockIdx.x;  // = b * Hkv + h
  const int cidx = CLUSTER ? (int)(blockIdx.x / 8) % cl.C : 0;  // this block's place among the unit's blocks
  if constexpr (CLUSTER) {
    if (unit >= cl.units) return;  // (padding of the launch: the unit's whole cluster leaves)
  }
  const int h = unit % Hkv;
  const size_t head0 = (size_t)unit * G;
  const int S = seq_rows(rag, unit / Hkv, S_max);
  const int k = seq_keep(rag, unit / Hkv, k_max, S);
  const int per_thread = gqa_keys_per_thread(L_max, THREADS);
  // the rows this block scores and attends over: [row0, row1)
  const int L = CLUSTER ? gqa_slice_rows(S, cl.C) : S;
  const int row0 = CLUSTER ? min(cidx * L, S) : 0;
  const int row1 = CLUSTER ? min(row0 + L, S) : S;
  // a launch that gave up earlier on this workspace left arrival flags behind (only a workspace
  // that is not cleared in front of every launch can show this): then this launch must not trust them
  bool poisoned = false;
  if constexpr (CLUSTER) {
    if (threadIdx.x == 0) poisoned = cluster_load_u32(cl.error) != 0u;
  }

  LOKI_STAMP(0);
#ifdef LOKI_PHASE_TIMING
  // where the block runs: XCC_ID (hardware register 20) above HW_ID (register 4: CU in bits 8-11,
  // shader array bit 12, shader engine bits 13-15)
  if (threadIdx.x == 0 && blockIdx.x < 8192)
    g_phase_ts[blockIdx.x * kPhaseSlots + 15] =
        ((unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32) |
        (unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 4);
#endif
  resident_select_clear<THREADS>(s_sel);  // covered by the barriers of the next stages

  // Loads return in the order they were issued, so they are issued in the order their results
  // are needed: the queries, this thread's entries of P_h, then the first slab loads, which need
  // no query and stay in flight during the rotation (issued first, they would hold P_h back
  // behind the whole chip's first burst of slab rows).
  constexpr int kDepth = LOKI_GQA_SCORE_DEPTH(NCH);
  constexpr int kQPerThread = (G * kD + THREADS - 1) / THREADS;
  using Rows = std::conditional_t<PAGED, PagedRows, ContiguousRows>;
  Rows slab;
  if constexpr (PAGED) {
    // the sequence's page list, clamped into the pool; readable after the first barrier below
    if (tid < kGqaMaxPages && tid < pg.pages_per_seq)
      s_pages[tid] = min(max(pg.table[(size_t)(unit / Hkv) * pg.pages_per_seq + tid], 0), pg.n_pages - 1);
    slab = PagedRows{reinterpret_cast<const char*>(klo) + score_mfma_chunk_bytes<NCH>(), (size_t)(d * 2),
                     s_pages, pg.lg_rows, Hkv, h};
  } else {
    slab = score_mfma_contiguous<NCH>(reinterpret_cast<const char*>(klo) +
                                      (size_t)unit * S_cap * (size_t)(d * 2));
  }
  ScoreMfmaBufs<NCH, kDepth> sbufs;

  // ---- qhat = q P_h for the G heads, with the association every path uses (8 parts of 16 terms,
  // parts added in order): wave w owns parts w PPW .. w PPW + PPW - 1, lane l columns 2l, 2l+1 ----
  // With ap.k_new the block also rotates the unit's new key, as one more vector through the
  // same partial sums, and writes it (rounded to storage) with the new value into row S - 1 of
  // the unit's cache before it scores (Algorithm 1 lines 3-4).  The block's own later reads of
  // that row go through the same L1 and see it after the barrier; no other block reads this
  // unit's rows.
  // (CLUSTER: by the block whose slice holds row S - 1)
  const bool app = ap.k_new != nullptr && (!CLUSTER || (S - 1 >= row0 && S - 1 < row1));
  {
    float qv[kQPerThread];
#pragma unroll
    for (int j = 0; j < kQPerThread; ++j) {
      const int i = tid + j * THREADS;
      qv[j] = BF16::load1(q + head0 * kD + (i < G * kD ? i : 0));
    }
    // (no branch around the loads: without a new key they read the first query again)
    const uint16_t* kn_src = app ? static_cast<const uint16_t*>(ap.k_new) + (size_t)unit * kD : q + head0 * kD;
    const uint16_t* vn_src = app ? static_cast<const uint16_t*>(ap.v_new) + (size_t)unit * kD : q + head0 * kD;
    const float kn_mine = BF16::load1(kn_src + (tid & (kD - 1)));
    const uint16_t vn_mine = vn_src[tid & (kD - 1)];
    float2 pv[PPW][kRotPartLen];
    const float* Ph = P + (size_t)h * kD * kD + 2 * lane;
#pragma unroll
    for (int pp = 0; pp < PPW; ++pp)
#pragma unroll
      for (int ii = 0; ii < kRotPartLen; ++ii)
        pv[pp][ii] = *reinterpret_cast<const float2*>(Ph + (size_t)((wave * PPW + pp) * kRotPartLen + ii) * kD);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (!PAGED) score_mfma_prefetch<NCH, kWaves, kDepth>(slab, row0, row1, sbufs);
#pragma unroll
    for (int j = 0; j < kQPerThread; ++j) {
      const int i = tid + j * THREADS;
      if (i < G * kD) s_q[i] = qv[j];
    }
    if (tid < kD) s_q[G * kD + tid] = kn_mine;
    __syncthreads();
    if constexpr (PAGED) score_mfma_prefetch<NCH, kWaves, kDepth>(slab, row0, row1, sbufs);  // the page list is in LDS now
#pragma unroll
    for (int g = 0; g < G + 1; ++g)
      if (g < G || app)  // (uniform)
#pragma unroll
      for (int pp = 0; pp < PPW; ++pp) {
        const int part = wave * PPW + pp;
        float a0 = 0.f, a1 = 0.f;
#pragma unroll
        for (int i4 = 0; i4 < kRotPartLen; i4 += 4) {
          const float4 qq = *reinterpret_cast<const float4*>(&s_q[g * kD + part * kRotPartLen + i4]);
          a0 = fmaf(qq.x, pv[pp][i4 + 0].x, a0);
          a1 = fmaf(qq.x, pv[pp][i4 + 0].y, a1);
          a0 = fmaf(qq.y, pv[pp][i4 + 1].x, a0);
          a1 = fmaf(qq.y, pv[pp][i4 + 1].y, a1);
          a0 = fmaf(qq.z, pv[pp][i4 + 2].x, a0);
          a1 = fmaf(qq.z, pv[pp][i4 + 2].y, a1);
          a0 = fmaf(qq.w, pv[pp][i4 + 3].x, a0);
          a1 = fmaf(qq.w, pv[pp][i4 + 3].y, a1);
        }
        *reinterpret_cast<float2*>(&s_part[(g * kRotParts + part) * kD + 2 * lane]) = make_float2(a0, a1);
      }
    __syncthreads();
    size_t new_row;
    if constexpr (PAGED) new_row = (size_t)slab.pool_row(S - 1);
    else new_row = (size_t)unit * S_cap + (size_t)(S - 1);
    for (int i = tid; i < (G + (app ? 1 : 0)) * kD; i += THREADS) {
      const int g = i / kD, j = i % kD;
      float sum = 0.f;
#pragma unroll
      for (int pp = 0; pp < kRotParts; ++pp) sum += s_part[(g * kRotParts + pp) * kD + j];
      if (g < G) {
        s_qhat[g][j] = sum;
      } else {  // the new key: columns < d to the low-rank slab, the rest to the residual slab
        uint16_t* dst = j < d ? const_cast<uint16_t*>(klo) + new_row * d + j
                              : const_cast<uint16_t*>(khi) + new_row * (kD - d) + (j - d);
        BF16::store1(dst, sum);
      }
    }
    if (app && tid >= THREADS - kD)  // the new value, by the last 128 threads (tid % 128 = column)
      const_cast<uint16_t*>(v)[new_row * kD + (tid & (kD - 1))] = vn_mine;
    __syncthreads();  // s_qhat complete; the partial sums are dead, the region turns into the scores
    // the loads put in flight before the rotation may have read row S - 1 before it was written
    constexpr int kPrefRows = 2 * kWaves * ScoreMfmaGeom<NCH>::RPS * ScoreMfmaBufs<NCH, kDepth>::UH;
    if (app && S - 1 - row0 < kPrefRows) score_mfma_prefetch<NCH, kWaves, kDepth>(slab, row0, row1, sbufs);
  }
  LOKI_STAMP(1);

  // ---- approximate scores: the key of every row's group maximum into LDS ----------------------
  // qhat is the A operand and the row tile the B operand, so a lane holds one row and four heads:
  // the maximum over the group is taken in registers (G = 8: one exchange between the lanes
  // that hold heads 0-3 and 4-7).  The first counting pass of the selection rides along: the
  // leading 11 bits of every row's key go into the histogram while the next rows' loads are in
  // flight.
  {
    const bool head_ok = r16 < G;
    const int kgrp = lane >> 4;
    bf16x8_t bq[ScoreMfmaGeom<NCH>::NB][3];
    score_mfma_operands<NCH>(s_qhat[head_ok ? r16 : 0], head_ok, bq);
    score_mfma_rows<NCH, kWaves, kDepth, true>(
        slab, row0, row1, bq, sbufs, [&](int rowbase_a, const f32x4_t& acc_a, int rowbase_b, const f32x4_t& acc_b) {
          // lanes 0-15: the group maximum of tile a's rows, lanes 16-31: of tile b's
          const float m = group_max_pair<G>(acc_a, acc_b);
          const int row = (kgrp == 0 ? rowbase_a : rowbase_b) + r16;
          if (kgrp < 2 && row < row1) {
            const uint32_t key = float_to_key(m);
            s_key[padded_pos(row - row0)] = key;
            atomicAdd(&s_sel.hist[0][key >> 21], 1u);
          }
        });
  }
  __syncthreads();
  LOKI_STAMP(2);

  // ---- top-k in LDS -----------------------------------------------------------------------------
  int32_t* gidx = out_idx ? out_idx + (size_t)unit * k_max : nullptr;
  if (gidx && cidx == 0)
    for (int i = k + tid; i < k_max; i += THREADS) gidx[i] = -1;  // a sequence keeping fewer rows
  constexpr int kCandCap = Lds::kCandCap;  // candidates resolved from a compact list (else: all keys)
  // what the stage leaves: s_idx[0, n_list) = this block's selected rows as two ascending runs,
  // [0, n_def) and [n_def, n_list); gidx_base = selected rows of the unit below this block's
  int n_list = k, n_def = 0, gidx_base = 0;
  if constexpr (CLUSTER) {
    const int C = cl.C;
    const int n = row1 - row0;
    uint32_t* counter = cl.counters + (size_t)unit * kClusterCounterStride;
    const __amdgpu_buffer_rsrc_t xh = cluster_buffer(cl.xhist, cl.xhist_bytes);
    const uint32_t round_bytes = (uint32_t)(C * THREADS * kClusterSlotBytes);
    const uint32_t xh_unit = (uint32_t)unit * kClusterRounds * round_bytes;
    int32_t* s_cpos = reinterpret_cast<int32_t*>(dyn_smem + Lds::cand_offset(L_max));  // behind the keys
    const uint32_t* run = s_key + padded_pos(tid * per_thread);  // this thread's keys (select_impl.h)
    const uint32_t vmask = contiguous_valid_mask(n, per_thread);
    // The threshold key is fixed digit by digit (11 + 11 + 10 bits, as in select_impl.h), each
    // digit by one histogram exchange between the unit's blocks; the first digit's histogram was
    // counted while scoring.  As soon as the rows that agree with the threshold so far are few
    // enough, they are ranked directly instead (below).
    uint32_t prefix = 0, rem = (uint32_t)k, meet = 0;
    uint32_t own_above = 0, lower_above = 0, own_inbin = 0, lower_inbin = 0, total_inbin = 0;
    int shift = 32;
    bool ok = true;
#pragma unroll 1
    for (int level = 0; level < kClusterRounds; ++level) {
      const int bits = level < 2 ? 11 : 10;
      if (level > 0) {
        for (int i = tid; i < 2048; i += THREADS) s_sel.hist[0][i] = 0u;  // (read for the last time inside the round)
        __syncthreads();
#pragma unroll
        for (int e = 0; e < KPT; ++e) {
          const uint32_t x = run[e];
          if (((vmask >> e) & 1u) && (x >> shift) == prefix)
            atomicAdd(&s_sel.hist[0][(x >> (shift - bits)) & ((1u << bits) - 1u)], 1u);
        }
        __syncthreads();
      }
      shift -= bits;
      ++meet;
      ok = cluster_hist_round<THREADS>(s_sel.hist[0], xh, xh_unit + (uint32_t)level * round_bytes, C, cidx, counter,
                                       meet, rem, cl.spin_limit, poisoned, s_sel.wave[0], s_cl);
      if (!ok) break;
      const ClusterRound r = cluster_round_result(s_cl, C, cidx);
      prefix = (prefix << bits) | r.bin;
      rem = r.rem;
      own_above += r.own_above;
      lower_above += r.lower_above;
      own_inbin = r.own_inbin;
      lower_inbin = r.lower_inbin;
      total_inbin = r.total_inbin;
      if (total_inbin <= (uint32_t)kCandCap) break;
    }
    LOKI_STAMP(11);
    if (ok && shift > 0) {
      // Rows above the threshold's leading digits are certain: straight into the list.  The rows
      // that share them are the candidates: their remaining key bits go to the unit's candidate
      // array (block after block, so it is in position order), their positions stay here.
      const __amdgpu_buffer_rsrc_t xc = cluster_buffer(cl.xcand, cl.xcand_bytes);
      const uint32_t xc_unit = (uint32_t)unit * (uint32_t)kCandCap * 4u;
      uint32_t* xc_words = cl.xcand + (size_t)unit * kCandCap;
      const uint32_t low_mask = (1u << shift) - 1u;
      contiguous_partition<THREADS, KPT>(
          s_key, n, per_thread, shift, prefix, s_sel.wave[0], [&](int rank, int pos) { s_idx[rank] = row0 + pos; },
          [&](int rank, int pos, uint32_t kk) {
            cluster_store_u32(xc_words + lower_inbin + rank, kk & low_mask);
            s_cpos[rank] = row0 + pos;
          });
      for (int i = tid; i < 2048; i += THREADS) s_sel.hist[0][i] = 0u;  // (read for the last time inside the round)
      if (tid == 0) s_cl.red[0] = s_cl.red[1] = 0u;
      ++meet;
      ok = cluster_arrive_and_wait(counter, C, cidx, meet, cl.spin_limit, poisoned, s_cl);
      LOKI_STAMP(4);
      if (ok) {
        // every block ranks all candidates (on their remaining bits, moved to the top of the
        // word) and finds the same threshold
        constexpr int CPT = Lds::kCandPerThread;
        static_assert(CPT % 4 == 0, "candidates are read four at a time");
        uint32_t ck[CPT], vm = 0;
        const int c0 = resident_pos0(CPT);
#pragma unroll
        for (int j = 0; j < CPT / 4; ++j) {
          const int ci = c0 + 256 * j;  // the layout resident_compact emits in: 4 consecutive candidates
          const cluster_u32x4 w = cluster_load_x4(xc, xc_unit + (uint32_t)min(ci, kCandCap - 4) * 4u);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const bool in = (uint32_t)(ci + e) < total_inbin;
            ck[4 * j + e] = in ? (w[e] << (32 - shift)) : 0u;
            vm |= (in ? 1u : 0u) << (4 * j + e);
          }
        }
        uint32_t Tp, need_eq;
        resident_threshold<THREADS, CPT>(ck, vm, rem, s_sel, Tp, need_eq);
        LOKI_STAMP(12);
        // candidates above / equal to the threshold in the blocks before this one and in this one
        uint32_t cnt_lower = 0, cnt_own = 0;
#pragma unroll
        for (int e = 0; e < CPT; ++e) {
          const uint32_t ci = (uint32_t)(c0 + 256 * (e / 4) + (e % 4));
          const uint32_t one = ((vm >> e) & 1u) ? ((ck[e] > Tp ? 1u : 0u) | (ck[e] == Tp ? 0x10000u : 0u)) : 0u;
          cnt_lower += ci < lower_inbin ? one : 0u;
          cnt_own += (ci >= lower_inbin && ci < lower_inbin + own_inbin) ? one : 0u;
        }
        cluster_block_add(cnt_lower, s_cl, 0);
        cluster_block_add(cnt_own, s_cl, 1);
        __syncthreads();
        const uint32_t lower_gt = s_cl.red[0] & 0xffffu, lower_eq = s_cl.red[0] >> 16;
        const uint32_t own_gt = s_cl.red[1] & 0xffffu, own_eq = s_cl.red[1] >> 16;
        const uint32_t base_lower = lower_gt + min(lower_eq, need_eq);  // chosen candidates before this block's
        const uint32_t take_eq = min(own_eq, need_eq > lower_eq ? need_eq - lower_eq : 0u);
        resident_compact<THREADS, CPT>(ck, vm, CPT, Tp, need_eq, 0u, 0u, s_sel.wave[0], s_sel.wave[1],
                                       [&](int rank, int ci, float) {
                                         const uint32_t local = (uint32_t)ci - lower_inbin;
                                         if (local < own_inbin)
                                           s_idx[own_above + ((uint32_t)rank - base_lower)] = s_cpos[local];
                                       });
        n_def = (int)own_above;
        n_list = (int)(own_above + own_gt + take_eq);
        gidx_base = (int)(lower_above + base_lower);
      }
    } else if (ok) {
      // all 32 bits are fixed (long runs of equal scores): the rows equal to the threshold are taken
      // in position order, so a block takes what the blocks before it leave of the rem needed
      const uint32_t take_eq = min(own_inbin, rem > lower_inbin ? rem - lower_inbin : 0u);
      contiguous_partition<THREADS, KPT>(
          s_key, n, per_thread, 0, prefix, s_sel.wave[0], [&](int rank, int pos) { s_idx[rank] = row0 + pos; },
          [&](int rank, int pos, uint32_t) {
            if ((uint32_t)rank < take_eq) s_idx[own_above + rank] = row0 + pos;
          });
      n_def = (int)own_above;
      n_list = (int)(own_above + take_eq);
      gidx_base = (int)(lower_above + min(lower_inbin, rem));
    }
    if (!ok) {
      // the other blocks of the unit did not show up in time: say so and leave a result that
      // cannot be mistaken for one (all threads take this branch together)
      if (tid == 0) cluster_store_u32(cl.error, 1u);
      for (int i = tid; i < G * kD; i += THREADS) out[head0 * kD + i] = 0x7fc0u;  // NaN
      return;
    }
  } else {
  // The histogram of the leading 11 key bits is complete: find the bin that holds the k-th
  // largest score.  Rows in higher bins are selected for certain (n_def of them); the rows
  // inside the bin are the candidates among which the exact threshold is found.
  resident_find_bin<THREADS>(s_sel, 0, (uint32_t)k);
  const uint32_t bin1 = s_sel.out[0][0], rem1 = s_sel.out[0][1];
  const uint32_t n_cand = s_sel.hist[0][bin1];
  n_def = k - (int)rem1;
  uint32_t* s_ckey = reinterpret_cast<uint32_t*>(dyn_smem + Lds::cand_offset(S_max));  // behind the keys
  int32_t* s_cpos = reinterpret_cast<int32_t*>(s_ckey + kCandCap);
  LOKI_STAMP(11);
  if (n_cand <= (uint32_t)kCandCap) {
    // certain rows straight into the list, the bin's rows into the candidate list
    contiguous_partition<THREADS, KPT>(
        s_key, S, per_thread, 21, bin1, s_sel.wave[0], [&](int rank, int pos) { s_idx[rank] = pos; },
        [&](int rank, int pos, uint32_t kk) {
          s_ckey[rank] = kk;
          s_cpos[rank] = pos;
        });
    for (int i = tid; i < 2048; i += THREADS) s_sel.hist[0][i] = 0u;  // everyone has read n_cand
    __syncthreads();
    LOKI_STAMP(13);
    // exact threshold among the candidates (they agree on the leading 11 bits: rank on the
    // remaining 21, moved to the top of the word) and ordered emission of the rem1 best
    constexpr int CPT = Lds::kCandPerThread;
    uint32_t ck[CPT], vm = 0;
    const int c0 = resident_pos0(CPT);
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
      const int ci = c0 + 256 * (e / 4) + (e % 4);  // the layout resident_compact emits in
      const bool ok = (uint32_t)ci < n_cand;
      ck[e] = ok ? (s_ckey[ci] << 11) : 0u;
      vm |= (ok ? 1u : 0u) << e;
    }
    uint32_t Tp, need_eq;
    resident_threshold<THREADS, CPT>(ck, vm, rem1, s_sel, Tp, need_eq);
    resident_compact<THREADS, CPT>(ck, vm, CPT, Tp, need_eq, 0u, 0u, s_sel.wave[0], s_sel.wave[1],
                                   [&](int rank, int local, float) { s_idx[n_def + rank] = s_cpos[local]; });
  } else {
    // long runs of (nearly) equal scores: the plain selection over all keys, held in registers;
    // the list is again two ascending runs: the keys above the threshold, then the first
    // need_eq keys equal to it
    uint32_t key[KPT];
    uint32_t valid_mask;
    contiguous_load_keys<KPT>(s_key, S, per_thread, key, valid_mask);
    __syncthreads();  // everyone has read n_cand
    for (int i = tid; i < 2048; i += THREADS) s_sel.hist[0][i] = 0u;
    __syncthreads();
    uint32_t T, need_eq;
    resident_threshold<THREADS, KPT>(key, valid_mask, (uint32_t)k, s_sel, T, need_eq);
    n_def = k - (int)need_eq;
    __syncthreads();  // s_sel.wave is free again
    contiguous_partition<THREADS, KPT>(
        s_key, S, per_thread, 0, T, s_sel.wave[0], [&](int rank, int pos) { s_idx[rank] = pos; },
        [&](int rank, int pos, uint32_t) {
          if (rank < (int)need_eq) s_idx[n_def + rank] = pos;
        });
  }
  }
  __syncthreads();  // the index list is complete; the scores are dead, the region turns into value tiles
  LOKI_STAMP(6);
  if (gidx) {
    // the list holds the certain rows (ascending) followed by the chosen candidates (ascending);
    // the caller's copy is the merge of the two (CLUSTER: behind the rows of the blocks before)
    const int n_chosen = n_list - n_def;
    for (int i = tid; i < n_list; i += THREADS) {
      const int pos = s_idx[i];
      const bool certain = i < n_def;
      const int32_t* other = certain ? s_idx + n_def : s_idx;
      int lo = 0, hi = certain ? n_chosen : n_def;
      while (lo < hi) {  // entries of the other run below pos
        const int mid = (lo + hi) >> 1;
        if (other[mid] < pos) lo = mid + 1;
        else hi = mid;
      }
      gidx[gidx_base + (certain ? i : i - n_def) + lo] = pos;
    }
  }

  if constexpr (PAGED) {
    // the attention stage addresses the pools from their start: positions -> pool rows
    __syncthreads();  // the merge above has read the positions
    for (int i = tid; i < n_list; i += THREADS) s_idx[i] = (int32_t)slab.pool_row(s_idx[i]);
    __syncthreads();
  }

  // ---- exact attention over the selected rows, all G heads ---------------------------------------
  {
    const bool head_ok = r16 < G;
    am_bf16x8_t bq[4][2];
    am_query_operands<4, 2>(s_qhat[head_ok ? r16 : 0], head_ok, kD, bq);
    const AmAddr<4> ad = am_make_addr<4, false>(klo, khi, v, PAGED ? (size_t)0 : (size_t)unit, S_cap, d);
    AmState st;
    st.init();
    am_attend_rows<true, 4, 2, kWaves>(ad, bq, s_idx, 0, n_list, s_stage + (size_t)wave * kAmStageBytes, st);
    __syncthreads();  // every wave is done with its value tiles: the region turns into the merge
    LOKI_STAMP(7);
    am_publish<G, kWaves>(st, s_merge);
  }
  for (int i = tid; i < G * kD; i += THREADS) {
    const int g = i / kD, col = i % kD;
    float mn, ls, os;
    attend_merged<kWaves, G>(s_merge, g, col, mn, ls, os);
    if constexpr (CLUSTER) {
      float* pr = cl.partial + ((head0 + g) * cl.C + cidx) * kPartialStride;
      store_shared_f32(pr + col, os, true);
      if (col == 0) {
        store_shared_f32(pr + kD, mn, true);
        store_shared_f32(pr + kD + 1, ls, true);
      }
    } else {
      out[(head0 + g) * kD + col] = BF16::round(os / ls);
    }
  }
  if constexpr (CLUSTER) {
    LOKI_STAMP(9);
    // the block of the unit that finishes last merges the slices' partial results
    uint32_t* ctl = cl.counters + (size_t)unit * kClusterCounterStride;
    if (splits_all_done(reinterpret_cast<int32_t*>(ctl + kClusterMax * kClusterFlagStride), cl.C)) {
      for (int i = tid; i < G * kD; i += THREADS)
        out[head0 * kD + i] = BF16::round(
            combine_splits<true>(cl.partial + (head0 + i / kD) * cl.C * kPartialStride, cl.C, i % kD));
      // every block of the unit is past its last wait and its flag store is acknowledged (it
      // took a ticket): leave the unit's flags and ticket at zero for the next launch
      if (tid <= kClusterMax) ctl[tid * kClusterFlagStride] = 0u;
    }
  }
  LOKI_STAMP(8);
}

}  // namespace loki
