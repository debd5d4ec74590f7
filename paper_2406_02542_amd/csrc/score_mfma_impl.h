// Low-rank scoring of a run of slab rows on the matrix cores (Algorithm 1 line 5 of
// arXiv 2406.02542 for several query heads that share one KV head's slab; bf16 cache):
//   scores[s, g] = sum_{j<d} Klo[s, j] qhat[g, j]
// A wave's 1 KiB load is directly the A operand of v_mfma_f32_16x16x32_bf16 (lane l supplies
// row l%16, columns 8*(l/16)..+7 — exactly one 16-byte chunk of a slab row) and qhat^T, padded
// to 16 heads, is the B operand.  qhat is fp32: it enters as three bf16 terms (value,
// remainder, remainder of the remainder = 24 significant bits), so the products are exact and
// a score differs from an fp32 vector dot product only by accumulation order; the bf16 keys
// are exact.  Shared by the stand-alone score kernel and the single-launch grouped-query kernel.
#pragma once

#include "score_impl.h"

namespace loki {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ inline void split_bf16x8(const float (&x)[8], bool active, bf16x8_t (&term)[3]) {
  uint32_t w[3][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t part[3][2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      float rest = active ? x[2 * i + e] : 0.f;
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        const uint16_t hb = BF16::round(rest);
        rest -= __uint_as_float((uint32_t)hb << 16);  // exact in fp32
        part[t][e] = hb;
      }
    }
#pragma unroll
    for (int t = 0; t < 3; ++t) w[t][i] = part[t][0] | (part[t][1] << 16);
  }
#pragma unroll
  for (int t = 0; t < 3; ++t)
    term[t] = __builtin_bit_cast(bf16x8_t, make_uint4(w[t][0], w[t][1], w[t][2], w[t][3]));
}

// NCH = 16-byte chunks per slab row (d = 8 * NCH).
template <int NCH>
struct ScoreMfmaGeom {
  static constexpr int RB = NCH <= 4 ? 4 / NCH : 1;   // 16-row blocks one load instruction covers
  static constexpr int NL = NCH <= 4 ? 1 : NCH / 4;   // load instructions per 16-row block
  static constexpr int NB = NCH <= 4 ? RB : NL;       // distinct B operands
  static constexpr int RPS = 16 * RB;                 // rows per wave step
};

// The B operands of head `r16` (this lane's column of the tile): qh points at that head's 128
// rotated-query values (global or LDS); lanes whose column holds no head pass active = false.
template <int NCH>
__device__ __forceinline__ void score_mfma_operands(const float* qh, bool active,
                                                    bf16x8_t (&bq)[ScoreMfmaGeom<NCH>::NB][3]) {
  const int kgrp = (threadIdx.x & 63) >> 4;
#pragma unroll
  for (int n = 0; n < ScoreMfmaGeom<NCH>::NB; ++n) {
    const int kbase = NCH <= 4 ? 8 * (kgrp % NCH) : 32 * n + 8 * kgrp;
    const bool act = active && (NCH <= 4 ? (kgrp / NCH == n) : true);
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = qh[kbase + e];
    split_bf16x8(x, act, bq[n]);
  }
}

// HEADS_IN_REGS epilogue for two tiles: acc_x holds heads 4 (lane / 16) .. + 3 of row lane % 16 of
// tile x.  Returns, in the lanes of 16-lane row 0, the maximum over the G heads of tile a's row and,
// in the lanes of row 1, that of tile b's row (rows 2 and 3 hold nothing of use).
// v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the even rows of
// its second: afterwards the first holds (a.row0, b.row0, ..) and the second (a.row1, b.row1, ..).
template <int G>
__device__ __forceinline__ float group_max_pair(const f32x4_t& acc_a, const f32x4_t& acc_b) {
  float ma = fmaxf(acc_a[0], acc_a[1]), mb = fmaxf(acc_b[0], acc_b[1]);
  if constexpr (G >= 4) {
    ma = fmaxf(ma, fmaxf(acc_a[2], acc_a[3]));
    mb = fmaxf(mb, fmaxf(acc_b[2], acc_b[3]));
  }
  typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
  const u32x2_t sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(ma), __float_as_uint(mb), false, false);
  if constexpr (G == 8) return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));  // heads 0-3 | 4-7
  else return __uint_as_float(sw[0]);  // the heads sit in row 0 alone
}

// The two register buffers of the tile loop (DEPTH / 2 16-byte loads per lane each).
template <int NCH, int DEPTH>
struct ScoreMfmaBufs {
  static constexpr int NL = ScoreMfmaGeom<NCH>::NL;
  static constexpr int UH = DEPTH / NL / 2;  // steps per buffer
  uint4 b0[UH][NL], b1[UH][NL];
};

// This lane's place in a wave step: its row inside the step and the byte offset of its 16-byte
// chunk inside a slab row.
template <int NCH>
__device__ __forceinline__ int score_mfma_row_in_step() {
  const int lane = threadIdx.x & 63;
  return NCH <= 4 ? (lane & 15) + 16 * ((lane >> 4) / NCH) : (lane & 15);
}
template <int NCH>
__device__ __forceinline__ int score_mfma_chunk_bytes() {
  const int kgrp = (threadIdx.x & 63) >> 4;
  return (NCH <= 4 ? (kgrp % NCH) : kgrp) * 16;
}
// `rows` maps a slab row to the address of this lane's chunk of it (ContiguousRows, or a paged
// cache's functor; the lane's chunk offset is part of its base).
template <int NCH, typename Rows>
struct ScoreMfmaLane {
  Rows rows;
  int row_in_step;
  __device__ __forceinline__ explicit ScoreMfmaLane(const Rows& r)
      : rows(r), row_in_step(score_mfma_row_in_step<NCH>()) {}
};
// rows one after the other from `slab` (the address row 0 would have)
template <int NCH>
__device__ __forceinline__ ContiguousRows score_mfma_contiguous(const char* slab) {
  return ContiguousRows{slab + score_mfma_chunk_bytes<NCH>(), (size_t)(NCH * 16)};
}

// One buffer's loads for the steps starting at row t0; rows past the end re-read the last row
// (no branch around a load).
template <int NCH, int WAVES, int UH, typename Rows>
__device__ __forceinline__ void score_mfma_load(const ScoreMfmaLane<NCH, Rows>& ln, int t0, int row_end,
                                                uint4 (&raw)[UH][ScoreMfmaGeom<NCH>::NL]) {
  constexpr int RPS = ScoreMfmaGeom<NCH>::RPS, NL = ScoreMfmaGeom<NCH>::NL;
#pragma unroll
  for (int u = 0; u < UH; ++u) {
    const char* p = ln.rows(min(t0 + u * WAVES * RPS + ln.row_in_step, row_end - 1));
#pragma unroll
    for (int j = 0; j < NL; ++j) raw[u][j] = load16(p + (size_t)j * 64);
  }
}

// Puts the loads of the first two buffers in flight; needs no query, so a caller can issue it
// ahead of the query rotation.  The scheduling barriers keep the two buffers' loads in issue
// order (buffer 0 before buffer 1, here as in the loop): loads return in order, and the wait in
// front of a buffer's first use can only leave the other buffer's loads in flight if they were
// issued after it on every path into the loop.
template <int NCH, int WAVES, int DEPTH, typename Rows>
__device__ __forceinline__ void score_mfma_prefetch(const Rows& rows, int row0, int row_end,
                                                    ScoreMfmaBufs<NCH, DEPTH>& bufs) {
  constexpr int UH = ScoreMfmaBufs<NCH, DEPTH>::UH;
  constexpr int kTrip = WAVES * ScoreMfmaGeom<NCH>::RPS * UH;
  const ScoreMfmaLane<NCH, Rows> ln(rows);
  const int t_first = row0 + (int)(threadIdx.x >> 6) * ScoreMfmaGeom<NCH>::RPS;
  score_mfma_load<NCH, WAVES, UH>(ln, t_first, row_end, bufs.b0);
  __builtin_amdgcn_sched_barrier(0);
  score_mfma_load<NCH, WAVES, UH>(ln, t_first + kTrip, row_end, bufs.b1);
  __builtin_amdgcn_sched_barrier(0);
}

// Scores rows [row0, row_end) with the block's WAVES waves; `bufs` holds the first two buffers
// (score_mfma_prefetch with the same arguments).  `rows` maps a row to this lane's chunk of it
// (score_mfma_contiguous for rows that follow each other in memory, 16 NCH bytes each); emit(rowbase, acc) is called by every lane with acc[i] =
// score of head (lane % 16) at row rowbase + i, rowbase = ... + 4 (lane / 16); rows at or past
// row_end carry the values of the last row and must not be used.  A buffer is refilled right
// after it is consumed, so that a wave always has loads in flight while it computes.
// DEPTH = 16-byte loads a lane keeps in flight (both buffers together).
// HEADS_IN_REGS: the two operands trade places (qhat is the A operand, the row tile the B
// operand), so that the accumulator holds the scores of ONE row per lane and four heads per
// lane in its registers, and tiles are handed out in pairs: emit(rowbase_a, acc_a, rowbase_b,
// acc_b) gets acc_x[i] = score of head 4 (lane / 16) + i at row rowbase_x + lane % 16, rowbase_x a
// multiple of 16 (rowbase_b >= row_end when a buffer holds an odd number of tiles and the second
// one is missing).  A maximum over the heads of a group is then taken in registers instead of
// across lanes, and one exchange between 16-lane rows (group_max_pair) leaves the two tiles'
// results in different lanes, so that what follows — key, store, count — is done once for both.
template <int NCH, int WAVES, int DEPTH = 8, bool HEADS_IN_REGS = false, typename Rows, typename Emit>
__device__ __forceinline__ void score_mfma_rows(const Rows& rows, int row0, int row_end,
                                                const bf16x8_t (&bq)[ScoreMfmaGeom<NCH>::NB][3],
                                                ScoreMfmaBufs<NCH, DEPTH>& bufs, Emit emit) {
  using Gm = ScoreMfmaGeom<NCH>;
  constexpr int RB = Gm::RB, NL = Gm::NL, RPS = Gm::RPS;
  constexpr int UH = ScoreMfmaBufs<NCH, DEPTH>::UH;
  constexpr int kTrip = WAVES * RPS * UH;    // rows the block advances per buffer
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kgrp = lane >> 4;
  const ScoreMfmaLane<NCH, Rows> ln(rows);

  auto score_trip = [&](const uint4 (&raw)[UH][NL], int t0) {
    f32x4_t pend = {0.f, 0.f, 0.f, 0.f};  // HEADS_IN_REGS: the first tile of a pair
    int pend_row = 0;
#pragma unroll
    for (int u = 0; u < UH; ++u) {
      const int trow = t0 + u * WAVES * RPS;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
        if constexpr (NCH <= 4) {
          const bf16x8_t a = __builtin_bit_cast(bf16x8_t, raw[u][0]);
#pragma unroll
          for (int t = 2; t >= 0; --t)  // smallest terms first
            acc = HEADS_IN_REGS ? __builtin_amdgcn_mfma_f32_16x16x32_bf16(bq[rb][t], a, acc, 0, 0, 0)
                                : __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bq[rb][t], acc, 0, 0, 0);
        } else {
#pragma unroll
          for (int j = 0; j < NL; ++j) {
            const bf16x8_t a = __builtin_bit_cast(bf16x8_t, raw[u][j]);
#pragma unroll
            for (int t = 2; t >= 0; --t)
              acc = HEADS_IN_REGS ? __builtin_amdgcn_mfma_f32_16x16x32_bf16(bq[j][t], a, acc, 0, 0, 0)
                                  : __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bq[j][t], acc, 0, 0, 0);
          }
        }
        if constexpr (HEADS_IN_REGS) {
          constexpr bool kPairs = (UH * RB) % 2 == 0;
          if constexpr (!kPairs) {
            emit(trow + 16 * rb, acc, 0x3fffffff, acc);
          } else if ((u * RB + rb) % 2 == 0) {
            pend = acc;
            pend_row = trow + 16 * rb;
          } else {
            emit(pend_row, pend, trow + 16 * rb, acc);
          }
        } else {
          emit(trow + 16 * rb + 4 * kgrp, acc);
        }
      }
    }
  };
  const int t_first = row0 + wave * RPS;
  for (int t0 = t_first; t0 < row_end; t0 += 2 * kTrip) {
    score_trip(bufs.b0, t0);
    score_mfma_load<NCH, WAVES, UH>(ln, t0 + 2 * kTrip, row_end, bufs.b0);
    __builtin_amdgcn_sched_barrier(0);
    score_trip(bufs.b1, t0 + kTrip);
    score_mfma_load<NCH, WAVES, UH>(ln, t0 + 3 * kTrip, row_end, bufs.b1);
    __builtin_amdgcn_sched_barrier(0);
  }
}

}  // namespace loki
