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
constexpr int kRotPartLen = kD / kRotParts;  // in a fixed order, whichever block computes it

// qhat[g][j] for j < ncols into s_qhat; THREADS threads.  Ends with a barrier.
template <typename T, int G, int THREADS>
__device__ inline void rotate_query_block(const typename T::store_t* __restrict__ q_heads,
                                          const float* __restrict__ Ph, int ncols,
                                          float (&s_q)[G][kD], float (&s_part)[G][kRotParts][kD],
                                          float (&s_qhat)[G][kD]) {
  const int tid = threadIdx.x;
  for (int i = tid; i < G * kD; i += THREADS) s_q[i / kD][i % kD] = T::load1(q_heads + i);
  __syncthreads();
  int ncol_pad = 1;
  while (ncol_pad < ncols) ncol_pad <<= 1;  // <= 128
  const int j = tid % ncol_pad;
  const int pg = tid / ncol_pad;
  const int ngroups = THREADS / ncol_pad;
  if (j < ncols) {
    for (int p = pg; p < kRotParts; p += ngroups) {
      float acc[G];
#pragma unroll
      for (int g = 0; g < G; ++g) acc[g] = 0.f;
#pragma unroll
      for (int ii = 0; ii < kRotPartLen; ++ii) {
        const int i = p * kRotPartLen + ii;
        const float pv = Ph[i * kD + j];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = fmaf(s_q[g][i], pv, acc[g]);
      }
#pragma unroll
      for (int g = 0; g < G; ++g) s_part[g][p][j] = acc[g];
    }
  }
  __syncthreads();
  for (int i = tid; i < G * ncols; i += THREADS) {
    const int g = i / ncols, jj = i % ncols;
    float s = 0.f;
#pragma unroll
    for (int p = 0; p < kRotParts; ++p) s += s_part[g][p][jj];
    s_qhat[g][jj] = s;
  }
  __syncthreads();
}

// Scores rows [row0, row_end) of one unit's low-rank slab with the block's WAVES waves.
// qr is this lane's slice of qhat (zero for lanes past the slab row's last chunk); `base`
// points at this lane's 16-byte chunk of slab row 0.  emit(row, scores[G]) is called once
// per row by the lane that ends up owning it.
template <typename T, int LPR, int G, int WAVES, typename Emit>
__device__ __forceinline__ void score_rows(const char* base, size_t row_bytes, bool cact,
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
          raw[tt][u] = (cact && row < row_end) ? load16(base + (size_t)row * row_bytes)
                                               : make_uint4(0, 0, 0, 0);
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

}  // namespace loki
