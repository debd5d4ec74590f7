// Query rotation and low-rank scoring (Algorithm 1 lines 3 and 5 of arXiv 2406.02542):
//   qhat = q P_h,   a[g, s] = sum_{j<d} qhat[g, j] * Klo[s, j]   (unscaled)
// Device functions shared by the stand-alone score kernel and the fused decode kernel.
// A wave reads 1 KiB of the slab per load instruction (64 lanes x 16 B, consecutive
// addresses); LPR consecutive lanes hold one row, multiply by their loop-invariant slice of
// qhat and are summed with DPP.
#pragma once

#include "common.h"

namespace loki {

constexpr int kRotParts = 8;                 // q P is summed as 8 partial sums of 16 terms each,
constexpr int kRotPartLen = kD / kRotParts;  // in a fixed order, whichever kernel computes it

// Where this lane's 16-byte chunk of slab row `row` lives: rows one after the other from `base`
// (this lane's chunk of row 0).  A paged cache supplies its own functor of the same shape.
struct ContiguousRows {
  const char* base;
  size_t row_bytes;
  __device__ __forceinline__ const char* operator()(int row) const {
    return base + (size_t)row * row_bytes;
  }
};

// Slab rows of a paged cache: the sequence's page list sits in LDS; a row's page is looked up
// per lane (rows past the end are clamped to the last row, which may lie in an earlier page).
struct PagedRows {
  const char* base;       // this lane's chunk of row 0 of the pool
  size_t row_bytes;
  const int32_t* pages;   // LDS: physical page of every logical page of the sequence
  int lg, Hkv, h;
  __device__ __forceinline__ long long pool_row(int row) const {
    return ((((long long)pages[row >> lg] * Hkv + h) << lg) | (long long)(row & ((1 << lg) - 1)));
  }
  __device__ __forceinline__ const char* operator()(int row) const {
    return base + pool_row(row) * (long long)row_bytes;
  }
};

// Scores rows [row0, row_end) of one unit's low-rank slab with the block's WAVES waves.
// qr is this lane's slice of qhat (zero for lanes past the slab row's last chunk); `rows`
// maps a row to this lane's 16-byte chunk of it.  emit(row, scores[G]) is called once
// per row by the lane that ends up owning it.
template <typename T, int LPR, int G, int WAVES, typename Rows, typename Emit>
__device__ __forceinline__ void score_rows(const Rows& rows, bool cact,
                                           const float (&qr)[G][T::EPC], int row0, int row_end,
                                           Emit emit) {
  constexpr int EPC = T::EPC;
  constexpr int RPI = 64 / LPR;              // rows one wave covers per load instruction
  constexpr int UNR = LPR < 8 ? LPR : 8;     // load instructions per tile kept in flight
  constexpr int TPI = LPR >= 8 ? 1 : 8 / LPR;  // 64-row tiles per loop trip (>= 8 loads in flight)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane % LPR, rsub = lane / LPR;

  for (int tile0 = row0 + wave * 64; tile0 < row_end; tile0 += WAVES * 64 * TPI) {
    float keep[TPI][G];
#pragma unroll
    for (int it0 = 0; it0 < LPR; it0 += UNR) {
      uint4 raw[TPI][UNR];
#pragma unroll
      for (int tt = 0; tt < TPI; ++tt)
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
          const int row = tile0 + tt * WAVES * 64 + (it0 + u) * RPI + rsub;
          raw[tt][u] = (cact && row < row_end) ? load16(rows(row)) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
      for (int tt = 0; tt < TPI; ++tt)
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
          float f[EPC];
          T::unpack(raw[tt][u], f);
#pragma unroll
          for (int g = 0; g < G; ++g) {
            float p = 0.f;
#pragma unroll
            for (int e = 0; e < EPC; ++e) p = fmaf(f[e], qr[g][e], p);
            p = group_allreduce_sum<LPR>(p);
            if (c == it0 + u) keep[tt][g] = p;
          }
        }
    }
    // lane now owns the score of row tile + c*RPI + rsub of each of its TPI tiles
#pragma unroll
    for (int tt = 0; tt < TPI; ++tt) {
      const int row = tile0 + tt * WAVES * 64 + c * RPI + rsub;
      if (row < row_end) emit(row, keep[tt]);
    }
  }
}

// ---- software-pipelined form (LPR <= 8) -----------------------------------------------------
// The loads of a trip are issued one trip ahead, and the first trip can be issued by the
// caller before it has qhat at all (e.g. ahead of the query rotation).  Loads never branch:
// rows past row_end re-read row row_end-1 and are simply not emitted, lanes past the slab
// row's last chunk read chunk 0 and multiply it by zero.
template <int LPR>
struct ScoreTrip {
  static_assert(LPR <= 8, "pipelined scoring keeps one load per chunk lane group");
  static constexpr int TPI = 8 / LPR;  // 64-row tiles per trip: 8 loads in flight per lane
  uint4 raw[TPI][LPR];
};

template <int LPR, int WAVES, typename Rows>
__device__ __forceinline__ void score_load_trip(const Rows& rows, int tile0, int row_end,
                                                ScoreTrip<LPR>& t) {
  constexpr int RPI = 64 / LPR;
  const int rsub = (threadIdx.x & 63) / LPR;
#pragma unroll
  for (int tt = 0; tt < ScoreTrip<LPR>::TPI; ++tt)
#pragma unroll
    for (int u = 0; u < LPR; ++u) {
      const int row = min(tile0 + tt * WAVES * 64 + u * RPI + rsub, row_end - 1);
      t.raw[tt][u] = load16(rows(row));
    }
}

// Scores one trip already (or about to be) in registers.
template <typename T, int LPR, int G, int WAVES, typename Emit>
__device__ __forceinline__ void score_trip(const ScoreTrip<LPR>& cur, const float (&qr)[G][T::EPC],
                                           int tile0, int row_end, Emit& emit) {
  constexpr int EPC = T::EPC;
  constexpr int RPI = 64 / LPR;
  constexpr int TPI = ScoreTrip<LPR>::TPI;
  const int lane = threadIdx.x & 63;
  const int c = lane % LPR, rsub = lane / LPR;
  float keep[TPI][G];
#pragma unroll
  for (int tt = 0; tt < TPI; ++tt)
#pragma unroll
    for (int u = 0; u < LPR; ++u) {
      float f[EPC];
      T::unpack(cur.raw[tt][u], f);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float p = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) p = fmaf(f[e], qr[g][e], p);
        p = group_allreduce_sum<LPR>(p);
        if (c == u) keep[tt][g] = p;
      }
    }
#pragma unroll
  for (int tt = 0; tt < TPI; ++tt) {
    const int row = tile0 + tt * WAVES * 64 + c * RPI + rsub;
    if (row < row_end) emit(row, keep[tt]);
  }
}

// `t0` and `t1` hold the trips of tile0 = row0 + wave*64 and tile0 + one stride, already in
// flight (the caller can issue them before it has qhat at all).  The two register buffers take
// turns (the loop body handles two trips), so two trips' loads stay in flight while a trip is
// scored and no buffer is ever copied; the loads past the last trip are clamped re-reads of
// the last row.
template <typename T, int LPR, int G, int WAVES, typename Rows, typename Emit>
__device__ __forceinline__ void score_rows_pipelined(const Rows& rows,
                                                     const float (&qr)[G][T::EPC], int row0,
                                                     int row_end, ScoreTrip<LPR>& t0,
                                                     ScoreTrip<LPR>& t1, Emit emit) {
  constexpr int kStride = WAVES * 64 * ScoreTrip<LPR>::TPI;
  const int wave = threadIdx.x >> 6;
  for (int tile0 = row0 + wave * 64; tile0 < row_end; tile0 += 2 * kStride) {
    score_trip<T, LPR, G, WAVES>(t0, qr, tile0, row_end, emit);
    score_load_trip<LPR, WAVES>(rows, tile0 + 2 * kStride, row_end, t0);
    score_trip<T, LPR, G, WAVES>(t1, qr, tile0 + kStride, row_end, emit);
    score_load_trip<LPR, WAVES>(rows, tile0 + 3 * kStride, row_end, t1);
  }
}

}  // namespace loki
