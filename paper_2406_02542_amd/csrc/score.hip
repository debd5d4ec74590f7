// Query rotation and low-rank scoring (Algorithm 1 lines 3 and 5 of arXiv 2406.02542) as
// stand-alone kernels for the split path, where the rows of a unit are spread over many
// blocks: qrot_kernel rotates every query once (qhat = q P_h, fp32, kept in the workspace for
// the attention stage too), and the score kernels stream the low-rank slab, one block scoring
// a run of rows of one (batch, KV head) unit for all G query heads of the group, so the slab
// is read once per unit.  (Where one block owns a whole unit the rotation is done inside that
// block instead: see fused.hip.)  A score block needs no LDS and no barrier: its slice of qhat
// goes straight to registers while the first slab loads are already in flight.
#include "score_impl.h"
#include "score_mfma_impl.h"

namespace loki {

// Block (unit, quarter) computes 32 columns of qhat for the unit's G query heads: thread
// (column j, part p) accumulates the 16 terms of part p, then the 8 parts are added in order —
// the same association as the fused decode kernel, so every path sees bit-identical qhat.
constexpr int kQrotCols = 32;

// APPEND: the unit's new key is rotated as one more vector beside the G queries and written,
// with the new value, into row seq_len-1 of the unit's cache; the kernels launched after this
// one see the row.
template <typename T, int G, bool APPEND>
__global__ __launch_bounds__(256) void qrot_kernel(const typename T::store_t* __restrict__ q,
                                                   const float* __restrict__ P,
                                                   float* __restrict__ qhat_out, int Hkv,
                                                   typename T::store_t* __restrict__ klo,
                                                   typename T::store_t* __restrict__ khi,
                                                   typename T::store_t* __restrict__ v, int S_max,
                                                   int S_cap, int d, Ragged rg, Append ap,
                                                   Paging pg, uint32_t* __restrict__ zero_words,
                                                   size_t n_zero) {
  using ST = typename T::store_t;
  constexpr int NV = G + (APPEND ? 1 : 0);
  // the chunk histograms the score kernel adds into (long sequences) start from zero
  if (zero_words != nullptr) {
    const size_t nthreads = (size_t)gridDim.x * gridDim.y * 256;
    for (size_t i = ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x; i < n_zero; i += nthreads)
      zero_words[i] = 0u;
  }
  __shared__ __align__(16) float s_q[NV][kD];
  __shared__ float s_part[NV][kRotParts][kQrotCols];
  const int tid = threadIdx.x;
  const int unit = blockIdx.x;
  const int h = unit % Hkv;
  const size_t head0 = (size_t)unit * G;
  const int jl = tid % kQrotCols, part = tid / kQrotCols;  // 8 parts of 16 terms
  const int j = blockIdx.y * kQrotCols + jl;
  const float* Ph = P + (size_t)h * kD * kD + j;

  float pv[kRotPartLen];
#pragma unroll
  for (int ii = 0; ii < kRotPartLen; ++ii) pv[ii] = Ph[(size_t)(part * kRotPartLen + ii) * kD];
  for (int i = tid; i < G * kD; i += 256) s_q[i / kD][i % kD] = T::load1(q + head0 * kD + i);
  size_t row = 0;
  if constexpr (APPEND) {
    if (tid < kD) s_q[G][tid] = T::load1(static_cast<const ST*>(ap.k_new) + (size_t)unit * kD + tid);
    row = (size_t)cache_row(pg, unit / Hkv / max(rg.queries, 1), h, Hkv, S_cap,
                            seq_rows(rg, unit / Hkv, S_max) - 1);
    if (blockIdx.y == 0 && tid >= kD)  // the value row is copied once per unit
      v[row * kD + (tid - kD)] = static_cast<const ST*>(ap.v_new)[(size_t)unit * kD + (tid - kD)];
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < NV; ++g) {
    float acc = 0.f;
#pragma unroll
    for (int i4 = 0; i4 < kRotPartLen; i4 += 4) {
      const float4 qq = *reinterpret_cast<const float4*>(&s_q[g][part * kRotPartLen + i4]);
      acc = fmaf(qq.x, pv[i4 + 0], acc);
      acc = fmaf(qq.y, pv[i4 + 1], acc);
      acc = fmaf(qq.z, pv[i4 + 2], acc);
      acc = fmaf(qq.w, pv[i4 + 3], acc);
    }
    s_part[g][part][jl] = acc;
  }
  __syncthreads();
  for (int i = tid; i < NV * kQrotCols; i += 256) {
    const int g = i / kQrotCols, jj = i % kQrotCols;
    float sum = 0.f;
#pragma unroll
    for (int pp = 0; pp < kRotParts; ++pp) sum += s_part[g][pp][jj];
    const int col = blockIdx.y * kQrotCols + jj;
    if (g < G) {
      qhat_out[(head0 + g) * kD + col] = sum;
    } else {
      ST* dst = col < d ? klo + row * d + col : khi + row * (kD - d) + (col - d);
      T::store1(dst, sum);
    }
  }
}

// Long sequences (hist_part != nullptr): the first counting pass of the selection rides along.
// The block counts the leading 11 bits of the key of every score it writes in LDS (16-bit
// counters, two bins per word: a block scores at most kHistChunk rows) and adds the counts into
// the histogram of the select chunk its rows belong to, hist_part[selecting head][chunk][2048];
// the host keeps a block inside one chunk.  The dynamic LDS holds kHistWords words per
// selecting head of the block (none without hist_part).
constexpr int kHistChunk = 16384;  // rows per select chunk (select.hip: kMbChunk)
constexpr int kHistWords = 1024;

__device__ __forceinline__ void hist_count(uint32_t* s_hist, float score) {
  const uint32_t bin = float_to_key(score) >> 21;
  atomicAdd(&s_hist[bin >> 1], 1u << ((bin & 1u) * 16));
}

template <int THREADS>
__device__ __forceinline__ void hist_flush(const uint32_t* s_hist, uint32_t* __restrict__ dst) {
  for (int i = threadIdx.x; i < kHistWords; i += THREADS) {
    const uint32_t w = s_hist[i];
    if (w & 0xffffu) atomicAdd(&dst[2 * i], w & 0xffffu);
    if (w >> 16) atomicAdd(&dst[2 * i + 1], w >> 16);
  }
}

template <typename T, int LPR, int G, bool GROUP_MAX>
__global__ __launch_bounds__(256) void score_kernel(
    const typename T::store_t* __restrict__ klo, const float* __restrict__ qhat,
    float* __restrict__ scores, int Hkv, int S_max, int S_cap, int d, int rows_per_block,
    Ragged rg, Paging pg, uint32_t* __restrict__ hist_part, int hist_chunks) {
  constexpr int EPC = T::EPC;
  constexpr int kSelHeads = GROUP_MAX ? 1 : G;  // selecting heads whose scores the block writes
  extern __shared__ uint32_t s_hist[];          // [kSelHeads][kHistWords] when hist_part is given
  const int tid = threadIdx.x;
  const int unit = blockIdx.y;
  const int S = seq_rows(rg, unit / Hkv, S_max);  // the score buffer keeps the stride S_max
  if ((int)blockIdx.x * rows_per_block >= S) return;
  const int head0 = unit * G;  // first query head of the group, flattened over batch
  const bool hist = hist_part != nullptr;
  if (hist) {
    for (int i = tid; i < kSelHeads * kHistWords; i += 256) s_hist[i] = 0u;
    __syncthreads();
  }

  const int lane = tid & 63;
  const int c = lane % LPR;
  const int nch = d / EPC;  // 16-byte chunks per slab row, <= LPR
  const bool cact = c < nch;
  float qr[G][EPC];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPC; ++e)
      qr[g][e] = cact ? qhat[(size_t)(head0 + g) * kD + c * EPC + e] : 0.f;

  const size_t row_bytes = (size_t)d * T::kBytes;
  const int row0 = blockIdx.x * rows_per_block;
  const int row_end = min(S, row0 + rows_per_block);
  // the block's rows are consecutive in memory (a paged cache: the host keeps a block inside a page)
  const long long row_shift =
      cache_row(pg, unit / Hkv / max(rg.queries, 1), unit % Hkv, Hkv, S_cap, row0) - row0;
  const char* base = reinterpret_cast<const char*>(klo) + row_shift * (long long)row_bytes +
                     (size_t)(cact ? c : 0) * 16;
  auto emit = [&](int row, const float (&sc)[G]) {
    if constexpr (GROUP_MAX) {
      float m = sc[0];
#pragma unroll
      for (int g = 1; g < G; ++g) m = fmaxf(m, sc[g]);
      scores[(size_t)unit * S_max + row] = m;
      if (hist) hist_count(s_hist, m);
    } else {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        scores[(size_t)(head0 + g) * S_max + row] = sc[g];
        if (hist) hist_count(s_hist + g * kHistWords, sc[g]);
      }
    }
  };
  const ContiguousRows rows{base, row_bytes};
  if constexpr (LPR <= 8) {
    // two trips of eight loads per lane in flight, refilled as they are consumed
    ScoreTrip<LPR> t0, t1;
    const int tile0 = row0 + (tid >> 6) * 64;
    score_load_trip<LPR, 4>(rows, tile0, row_end, t0);
    score_load_trip<LPR, 4>(rows, tile0 + 4 * 64 * ScoreTrip<LPR>::TPI, row_end, t1);
    score_rows_pipelined<T, LPR, G, 4>(rows, qr, row0, row_end, t0, t1, emit);
  } else {
    score_rows<T, LPR, G, 4>(rows, cact, qr, row0, row_end, emit);
  }
  if (hist) {
    __syncthreads();
    const size_t sel0 = GROUP_MAX ? (size_t)unit : (size_t)head0;
#pragma unroll
    for (int g = 0; g < kSelHeads; ++g)
      hist_flush<256>(s_hist + g * kHistWords,
                      hist_part + ((sel0 + g) * hist_chunks + row0 / kHistChunk) * 2048);
  }
}

// ---- matrix-core variant for grouped queries on a bf16 cache ----------------------------------
// With G > 1 query heads per KV head the scoring step is a small dense contraction per row tile,
// scores[s, g] = sum_j Klo[s, j] qhat[g, j], and the per-byte vector work of the kernel above
// grows with G until it, not HBM, sets the pace.  The tile loop is score_mfma_rows
// (score_mfma_impl.h); this kernel decides which heads form the 16 columns and where their
// scores go.
//
// NCH = 16-byte chunks per slab row (d = 8 * NCH).
// TILE: several new tokens per sequence (rg.queries = m > 1).  The m G query heads that read one
// KV head's slab form the 16 columns of the B operand, 16 / G tokens per block (blockIdx.z picks
// the tile of tokens, blockIdx.y the sequence and KV head), so the slab is read once per tile
// instead of once per token: [m G, d] x [d, S] as one contraction.  Token j only has scores for
// the rows of its own causal length; the block covers the longest length of its tile.
template <int NCH, int G, bool GROUP_MAX, bool TILE>
__global__ __launch_bounds__(256) void score_mfma_kernel(
    const uint16_t* __restrict__ klo, const float* __restrict__ qhat, float* __restrict__ scores,
    int Hkv, int S_max, int S_cap, int rows_per_block, Ragged rg, Paging pg,
    uint32_t* __restrict__ hist_part, int hist_chunks) {
  constexpr int kSelHeads = GROUP_MAX ? 1 : G;  // (histograms: one token per sequence only)
  extern __shared__ uint32_t s_hist[];          // [kSelHeads][kHistWords] when hist_part is given
  const int lane = threadIdx.x & 63;
  const int r16 = lane & 15;

  // column r16 of the tile: which query head it is, where its scores go, how many rows it sees
  int S;            // rows the block scores up to (uniform)
  int S_lane;       // rows head r16 has scores for
  bool head_ok;
  size_t head;      // row of qhat
  size_t score_row; // row of the score buffer
  int cache_b, hkv;
  if constexpr (TILE) {
    constexpr int QPT = 16 / G;  // tokens per tile
    const int m = rg.queries;
    const int bs = (int)blockIdx.y / Hkv, j0 = (int)blockIdx.z * QPT;
    hkv = (int)blockIdx.y % Hkv;
    cache_b = bs;
    const int j = j0 + r16 / G;
    head_ok = j < m;
    const int entry = bs * m + min(j, m - 1);
    head = ((size_t)entry * Hkv + hkv) * G + r16 % G;
    score_row = GROUP_MAX ? (size_t)entry * Hkv + hkv : head;
    S_lane = seq_rows(rg, entry, S_max);
    S = 0;
    for (int jj = j0; jj < min(j0 + QPT, m); ++jj) S = max(S, seq_rows(rg, bs * m + jj, S_max));
  } else {
    const int unit = blockIdx.y;
    hkv = unit % Hkv;
    cache_b = unit / Hkv;
    head_ok = r16 < G;
    head = (size_t)unit * G + (head_ok ? r16 : 0);
    score_row = GROUP_MAX ? (size_t)unit : head;
    S = S_lane = seq_rows(rg, cache_b, S_max);  // the score buffer keeps the stride S_max
  }
  if ((int)blockIdx.x * rows_per_block >= S) return;
  const bool hist = !TILE && hist_part != nullptr;
  if (hist) {
    for (int i = threadIdx.x; i < kSelHeads * kHistWords; i += 256) s_hist[i] = 0u;
    __syncthreads();
  }

  bf16x8_t bq[ScoreMfmaGeom<NCH>::NB][3];
  score_mfma_operands<NCH>(qhat + head * kD, head_ok, bq);

  const int row0 = blockIdx.x * rows_per_block;
  const int row_end = min(S, row0 + rows_per_block);
  // the block's rows are consecutive in memory (a paged cache: the host keeps a block inside a page)
  const long long row_shift = cache_row(pg, cache_b, hkv, Hkv, S_cap, row0) - row0;
  const int lane_end = min(row_end, S_lane);
  const char* slab = reinterpret_cast<const char*>(klo) + row_shift * (long long)(NCH * 16);
  const bool vec_ok = (S_max & 3) == 0;
  ScoreMfmaBufs<NCH, 8> bufs;
  const ContiguousRows slab_rows = score_mfma_contiguous<NCH>(slab);
  score_mfma_prefetch<NCH, 4, 8>(slab_rows, row0, row_end, bufs);
  if constexpr (GROUP_MAX && !TILE) {
    // One score per row, the maximum over the group: qhat is the A operand and the row tile the
    // B operand, so a lane holds one row and four heads in its registers and the maximum needs
    // no exchange between lanes but one, which also puts the results of two tiles side by side:
    // thirty-two lanes store the rows of two tiles.
    const int kgrp = lane >> 4;
    score_mfma_rows<NCH, 4, 8, true>(
        slab_rows, row0, row_end, bq, bufs,
        [&](int rowbase_a, const f32x4_t& acc_a, int rowbase_b, const f32x4_t& acc_b) {
          // lanes 0-15: the group maximum of tile a's rows, lanes 16-31: of tile b's
          const float m = group_max_pair<G>(acc_a, acc_b);
          const int row = (kgrp == 0 ? rowbase_a : rowbase_b) + r16;
          if (kgrp < 2 && row < lane_end) {
            scores[score_row * S_max + row] = m;
            if (hist) hist_count(s_hist, m);
          }
        });
  } else {
  score_mfma_rows<NCH, 4, 8>(slab_rows, row0, row_end, bq, bufs, [&](int rowbase, const f32x4_t& acc) {
    float v[4] = {acc[0], acc[1], acc[2], acc[3]};
    bool writer = head_ok;
    if constexpr (GROUP_MAX) {
      // the G heads of one token sit in G consecutive lanes
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = group_allreduce_max<G>(head_ok ? v[i] : -3.0e38f);
      writer = head_ok && (r16 % G == 0);
    }
    float* dst = scores + score_row * S_max + rowbase;
    if (writer && rowbase < lane_end) {
      if (vec_ok && rowbase + 3 < lane_end) {
        *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (rowbase + i < lane_end) dst[i] = v[i];
      }
      if (hist) {
        uint32_t* mine = s_hist + (GROUP_MAX ? 0 : r16) * kHistWords;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (rowbase + i < lane_end) hist_count(mine, v[i]);
      }
    }
  });
  }
  if (hist) {
    __syncthreads();
    const size_t sel0 = GROUP_MAX ? (size_t)blockIdx.y : (size_t)blockIdx.y * G;
#pragma unroll
    for (int g = 0; g < kSelHeads; ++g)
      hist_flush<256>(s_hist + g * kHistWords,
                      hist_part + ((sel0 + g) * hist_chunks + row0 / kHistChunk) * 2048);
  }
}

// tokens of one sequence that share a score block (TILE), and the blocks along z that takes
static int score_tile_tokens(const Shape& s) { return 16 / s.G; }

template <int NCH, int G, bool TILE>
static hipError_t launch_score_mfma_g(const Shape& s, int select_mode, const void* klo, float* scores,
                                      const float* qhat, uint32_t* hist_part, int hist_chunks,
                                      hipStream_t st) {
  const int m = TILE ? s.rg.queries : 1;
  const int nz = TILE ? (m + score_tile_tokens(s) - 1) / score_tile_tokens(s) : 1;
  Shape blocks = s;  // the grid's y*z extent stands in for the batch when the row block is sized
  blocks.B = s.B / m * nz;
  const int rpb = score_rows_per_block(blocks);
  dim3 grid((s.S + rpb - 1) / rpb, s.B / m * s.Hkv, nz);
  if (TILE) hist_part = nullptr;  // (several tokens per sequence keep the separate counting pass)
  if (select_mode == 1 && G > 1) {
    hipLaunchKernelGGL((score_mfma_kernel<NCH, G, (G > 1), TILE>), grid, dim3(256),
                       hist_part ? kHistWords * 4 : 0, st, static_cast<const uint16_t*>(klo), qhat,
                       scores, s.Hkv, s.S, s.S_cap, rpb, s.rg, s.pg, hist_part, hist_chunks);
  } else {
    hipLaunchKernelGGL((score_mfma_kernel<NCH, G, false, TILE>), grid, dim3(256),
                       hist_part ? G * kHistWords * 4 : 0, st, static_cast<const uint16_t*>(klo), qhat,
                       scores, s.Hkv, s.S, s.S_cap, rpb, s.rg, s.pg, hist_part, hist_chunks);
  }
  return hipGetLastError();
}

template <int NCH>
static hipError_t launch_score_mfma_n(const Shape& s, int select_mode, const void* klo, float* scores,
                                      const float* qhat, uint32_t* hist_part, int hist_chunks,
                                      hipStream_t st) {
  if (s.rg.queries > 1) {
    switch (s.G) {
      case 1: return launch_score_mfma_g<NCH, 1, true>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
      case 2: return launch_score_mfma_g<NCH, 2, true>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
      case 4: return launch_score_mfma_g<NCH, 4, true>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
      case 8: return launch_score_mfma_g<NCH, 8, true>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
      default: return hipErrorInvalidValue;
    }
  }
  switch (s.G) {
    case 2: return launch_score_mfma_g<NCH, 2, false>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
    case 4: return launch_score_mfma_g<NCH, 4, false>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
    case 8: return launch_score_mfma_g<NCH, 8, false>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
    default: return hipErrorInvalidValue;
  }
}

// bf16 cache, a power-of-two number of chunks per slab row, and at least two query heads that
// share a slab: 2..8 per KV head, or several new tokens per sequence.  With rows of 16 or 32
// bytes (d <= 16) a matrix instruction is spent on very few bytes and the vector kernel is the
// faster one when every head's score is written (d = 16, 4 heads per KV head, S = 131072: 39
// against 44 us; d = 8: 12 against 33 us); with one selection per group, where the tiles are
// finished in pairs in registers, 32-byte rows are level or slightly ahead (35 against 36 us).
static bool score_mfma_applies(const Shape& s, int select_mode) {
  const int nch = s.d / 8;
  const bool tile = s.rg.queries > 1;
  const bool shared = (s.G >= 2 || tile) && s.G <= 8;
  const bool wide_enough = nch > 2 || tile || (nch == 2 && select_mode == 1);
  return s.dtype == 1 && shared && s.d % 8 == 0 && (nch & (nch - 1)) == 0 && wide_enough;
}

static hipError_t launch_score_mfma(const Shape& s, int select_mode, const void* klo, float* scores,
                                    const float* qhat, uint32_t* hist_part, int hist_chunks,
                                    hipStream_t st) {
  switch (s.d / 8) {
    case 1: return launch_score_mfma_n<1>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
    case 2: return launch_score_mfma_n<2>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
    case 4: return launch_score_mfma_n<4>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
    case 8: return launch_score_mfma_n<8>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
    case 16: return launch_score_mfma_n<16>(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
    default: return hipErrorInvalidValue;
  }
}

template <typename T, int LPR, int G>
static hipError_t launch_score_g(const Shape& s, int select_mode, const void* q, const float* P,
                                 const void* klo, float* scores, float* qhat, uint32_t* hist_part,
                                 int hist_chunks, hipStream_t st) {
  using ST = typename T::store_t;
  const int rpb = score_rows_per_block(s);
  dim3 grid((s.S + rpb - 1) / rpb, s.B * s.Hkv);
  const bool gm = (select_mode == 1) && (G > 1);
  if (s.rg.queries > 1) hist_part = nullptr;  // (several tokens per sequence keep the separate counting pass)
  if (gm) {
    hipLaunchKernelGGL((score_kernel<T, LPR, G, (G > 1)>), grid, dim3(256),
                       hist_part ? kHistWords * 4 : 0, st, static_cast<const ST*>(klo), qhat, scores,
                       s.Hkv, s.S, s.S_cap, s.d, rpb, s.rg, s.pg, hist_part, hist_chunks);
  } else {
    hipLaunchKernelGGL((score_kernel<T, LPR, G, false>), grid, dim3(256),
                       hist_part ? G * kHistWords * 4 : 0, st, static_cast<const ST*>(klo), qhat, scores,
                       s.Hkv, s.S, s.S_cap, s.d, rpb, s.rg, s.pg, hist_part, hist_chunks);
  }
  return hipGetLastError();
}

template <typename T, int LPR>
static hipError_t launch_score_l(const Shape& s, int select_mode, const void* q, const float* P,
                                 const void* klo, float* scores, float* qhat, uint32_t* hist_part,
                                 int hist_chunks, hipStream_t st) {
  switch (s.G) {
    case 1: return launch_score_g<T, LPR, 1>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
    case 2: return launch_score_g<T, LPR, 2>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
    case 4: return launch_score_g<T, LPR, 4>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
    case 8: return launch_score_g<T, LPR, 8>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
    default: return hipErrorInvalidValue;
  }
}

template <typename T>
static hipError_t launch_score_t(const Shape& s, int select_mode, const void* q, const float* P,
                                 const void* klo, float* scores, float* qhat, uint32_t* hist_part,
                                 int hist_chunks, hipStream_t st) {
  const int nch = s.d / T::EPC;
  int lpr = 1;
  while (lpr < nch) lpr <<= 1;
  switch (lpr) {
    case 1: return launch_score_l<T, 1>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
    case 2: return launch_score_l<T, 2>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
    case 4: return launch_score_l<T, 4>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
    case 8: return launch_score_l<T, 8>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
    case 16: return launch_score_l<T, 16>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
    case 32:
      if constexpr (T::EPC == 4) return launch_score_l<T, 32>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

template <typename T, bool APPEND>
static hipError_t launch_qrot_t(const Shape& s, const void* q, const float* P, float* qhat, void* klo,
                                void* khi, void* v, uint32_t* zero_words, size_t n_zero, hipStream_t st) {
  using ST = typename T::store_t;
  const dim3 grid(s.B * s.Hkv, kD / kQrotCols), block(256);
#define LOKI_QROT(GV)                                                                            \
  hipLaunchKernelGGL((qrot_kernel<T, GV, APPEND>), grid, block, 0, st, static_cast<const ST*>(q), P, \
                     qhat, s.Hkv, static_cast<ST*>(klo), static_cast<ST*>(khi), static_cast<ST*>(v), \
                     s.S, s.S_cap, s.d, s.rg, s.ap, s.pg, zero_words, n_zero);                   \
  break
  switch (s.G) {
    case 1: LOKI_QROT(1);
    case 2: LOKI_QROT(2);
    case 4: LOKI_QROT(4);
    case 8: LOKI_QROT(8);
    default: return hipErrorInvalidValue;
  }
#undef LOKI_QROT
  return hipGetLastError();
}

hipError_t launch_qrot(const Shape& s, const void* q, const float* P, float* qhat, void* klo,
                       void* khi, void* v, uint32_t* zero_words, size_t n_zero, hipStream_t st) {
  if (s.ap.k_new != nullptr)
    return s.dtype == 0 ? launch_qrot_t<F32, true>(s, q, P, qhat, klo, khi, v, zero_words, n_zero, st)
                        : launch_qrot_t<BF16, true>(s, q, P, qhat, klo, khi, v, zero_words, n_zero, st);
  return s.dtype == 0 ? launch_qrot_t<F32, false>(s, q, P, qhat, klo, khi, v, zero_words, n_zero, st)
                      : launch_qrot_t<BF16, false>(s, q, P, qhat, klo, khi, v, zero_words, n_zero, st);
}

hipError_t launch_score(const Shape& s, int select_mode, const void* q, const float* P,
                        const void* klo, float* scores, float* qhat, uint32_t* hist_part,
                        int hist_chunks, hipStream_t st) {
  if (score_mfma_applies(s, select_mode))
    return launch_score_mfma(s, select_mode, klo, scores, qhat, hist_part, hist_chunks, st);
  return s.dtype == 0
             ? launch_score_t<F32>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st)
             : launch_score_t<BF16>(s, select_mode, q, P, klo, scores, qhat, hist_part, hist_chunks, st);
}

}  // namespace loki
