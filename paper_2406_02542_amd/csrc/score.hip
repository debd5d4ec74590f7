// Query rotation fused with low-rank scoring (Algorithm 1 lines 3 and 5 of arXiv 2406.02542):
//   qhat = q P_h,   a[g, s] = sum_{j<d} qhat[g, j] * Klo[s, j]   (unscaled)
// One block scores a run of rows of one (batch, KV head) unit for all G query heads of the
// group, so the slab is streamed once per unit.  A wave reads 1 KiB of the slab per load
// instruction (64 lanes x 16 B, consecutive addresses); LPR consecutive lanes hold one row,
// multiply by their loop-invariant slice of qhat and are summed with DPP.
#include "common.h"
#include "launch.h"

namespace loki {

constexpr int kRotParts = 8;                 // q P is summed as 8 partial sums of 16 terms each,
constexpr int kRotPartLen = kD / kRotParts;  // in a fixed order, whichever block computes it

// qhat[g][j] for j < ncols into s_qhat; 256 threads.
template <typename T, int G>
__device__ inline void rotate_query_block(const typename T::store_t* __restrict__ q_heads,
                                          const float* __restrict__ Ph, int ncols,
                                          float (&s_q)[G][kD], float (&s_part)[G][kRotParts][kD],
                                          float (&s_qhat)[G][kD]) {
  const int tid = threadIdx.x;
  for (int i = tid; i < G * kD; i += 256) s_q[i / kD][i % kD] = T::load1(q_heads + i);
  __syncthreads();
  int ncol_pad = 1;
  while (ncol_pad < ncols) ncol_pad <<= 1;  // <= 128
  const int j = tid % ncol_pad;
  const int pg = tid / ncol_pad;
  const int ngroups = 256 / ncol_pad;
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
  for (int i = tid; i < G * ncols; i += 256) {
    const int g = i / ncols, jj = i % ncols;
    float s = 0.f;
#pragma unroll
    for (int p = 0; p < kRotParts; ++p) s += s_part[g][p][jj];
    s_qhat[g][jj] = s;
  }
  __syncthreads();
}

template <typename T, int LPR, int G, bool GROUP_MAX>
__global__ __launch_bounds__(256) void score_kernel(
    const typename T::store_t* __restrict__ klo, const typename T::store_t* __restrict__ q,
    const float* __restrict__ P, float* __restrict__ scores, float* __restrict__ qhat_out,
    int Hkv, int S, int S_cap, int d, int rows_per_block) {
  constexpr int EPC = T::EPC;
  constexpr int RPI = 64 / LPR;              // rows one wave covers per load instruction
  constexpr int UNR = LPR < 8 ? LPR : 8;     // load instructions per tile kept in flight
  constexpr int TPI = LPR >= 8 ? 1 : 8 / LPR;  // 64-row tiles per loop trip (>= 8 loads in flight)

  __shared__ float s_q[G][kD];
  __shared__ float s_part[G][kRotParts][kD];
  __shared__ float s_qhat[G][kD];

  const int tid = threadIdx.x;
  const int unit = blockIdx.y;
  const int b = unit / Hkv, h = unit % Hkv;
  const int head0 = (b * Hkv + h) * G;  // first query head of the group, flattened over batch

  // Block 0 of a unit rotates all D columns and publishes qhat for the attention stage.
  const int ncols = (blockIdx.x == 0) ? kD : d;
  rotate_query_block<T, G>(q + (size_t)head0 * kD, P + (size_t)h * kD * kD, ncols, s_q, s_part,
                           s_qhat);
  if (blockIdx.x == 0) {
    for (int i = tid; i < G * kD; i += 256) qhat_out[(size_t)head0 * kD + i] = s_qhat[i / kD][i % kD];
  }

  const int lane = tid & 63, wave = tid >> 6;
  const int c = lane % LPR, rsub = lane / LPR;
  const int nch = d / EPC;  // 16-byte chunks per slab row, <= LPR
  const bool cact = c < nch;
  float qr[G][EPC];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPC; ++e) qr[g][e] = cact ? s_qhat[g][c * EPC + e] : 0.f;

  const size_t row_bytes = (size_t)d * T::kBytes;
  const char* base = reinterpret_cast<const char*>(klo) + (size_t)unit * S_cap * row_bytes +
                     (size_t)(cact ? c : 0) * 16;
  const int row0 = blockIdx.x * rows_per_block;
  const int row_end = min(S, row0 + rows_per_block);

  for (int tile0 = row0 + wave * 64; tile0 < row_end; tile0 += 4 * 64 * TPI) {
    float keep[TPI][G];
#pragma unroll
    for (int it0 = 0; it0 < LPR; it0 += UNR) {
      uint4 raw[TPI][UNR];
#pragma unroll
      for (int tt = 0; tt < TPI; ++tt)
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
          const int row = tile0 + tt * 256 + (it0 + u) * RPI + rsub;
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
      const int row = tile0 + tt * 256 + c * RPI + rsub;
      if (row < row_end) {
        if constexpr (GROUP_MAX) {
          float m = keep[tt][0];
#pragma unroll
          for (int g = 1; g < G; ++g) m = fmaxf(m, keep[tt][g]);
          scores[(size_t)unit * S + row] = m;
        } else {
#pragma unroll
          for (int g = 0; g < G; ++g) scores[(size_t)(head0 + g) * S + row] = keep[tt][g];
        }
      }
    }
  }
}

template <typename T, int LPR, int G>
static hipError_t launch_score_g(const Shape& s, int select_mode, const void* q, const float* P,
                                 const void* klo, float* scores, float* qhat, hipStream_t st) {
  using ST = typename T::store_t;
  const int rpb = score_rows_per_block(s);
  dim3 grid((s.S + rpb - 1) / rpb, s.B * s.Hkv);
  const bool gm = (select_mode == 1) && (G > 1);
  if (gm) {
    hipLaunchKernelGGL((score_kernel<T, LPR, G, (G > 1)>), grid, dim3(256), 0, st,
                       static_cast<const ST*>(klo), static_cast<const ST*>(q), P, scores, qhat,
                       s.Hkv, s.S, s.S_cap, s.d, rpb);
  } else {
    hipLaunchKernelGGL((score_kernel<T, LPR, G, false>), grid, dim3(256), 0, st,
                       static_cast<const ST*>(klo), static_cast<const ST*>(q), P, scores, qhat,
                       s.Hkv, s.S, s.S_cap, s.d, rpb);
  }
  return hipGetLastError();
}

template <typename T, int LPR>
static hipError_t launch_score_l(const Shape& s, int select_mode, const void* q, const float* P,
                                 const void* klo, float* scores, float* qhat, hipStream_t st) {
  switch (s.G) {
    case 1: return launch_score_g<T, LPR, 1>(s, select_mode, q, P, klo, scores, qhat, st);
    case 2: return launch_score_g<T, LPR, 2>(s, select_mode, q, P, klo, scores, qhat, st);
    case 4: return launch_score_g<T, LPR, 4>(s, select_mode, q, P, klo, scores, qhat, st);
    case 8: return launch_score_g<T, LPR, 8>(s, select_mode, q, P, klo, scores, qhat, st);
    default: return hipErrorInvalidValue;
  }
}

template <typename T>
static hipError_t launch_score_t(const Shape& s, int select_mode, const void* q, const float* P,
                                 const void* klo, float* scores, float* qhat, hipStream_t st) {
  const int nch = s.d / T::EPC;
  int lpr = 1;
  while (lpr < nch) lpr <<= 1;
  switch (lpr) {
    case 1: return launch_score_l<T, 1>(s, select_mode, q, P, klo, scores, qhat, st);
    case 2: return launch_score_l<T, 2>(s, select_mode, q, P, klo, scores, qhat, st);
    case 4: return launch_score_l<T, 4>(s, select_mode, q, P, klo, scores, qhat, st);
    case 8: return launch_score_l<T, 8>(s, select_mode, q, P, klo, scores, qhat, st);
    case 16: return launch_score_l<T, 16>(s, select_mode, q, P, klo, scores, qhat, st);
    case 32:
      if constexpr (T::EPC == 4) return launch_score_l<T, 32>(s, select_mode, q, P, klo, scores, qhat, st);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_score(const Shape& s, int select_mode, const void* q, const float* P,
                        const void* klo, float* scores, float* qhat, hipStream_t st) {
  return s.dtype == 0 ? launch_score_t<F32>(s, select_mode, q, P, klo, scores, qhat, st)
                      : launch_score_t<BF16>(s, select_mode, q, P, klo, scores, qhat, st);
}

}  // namespace loki
