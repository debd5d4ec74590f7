// Query rotation fused with low-rank scoring (Algorithm 1 lines 3 and 5 of arXiv 2406.02542)
// as a stand-alone kernel: one block scores a run of rows of one (batch, KV head) unit for
// all G query heads of the group, so the slab is streamed once per unit.
#include "score_impl.h"

namespace loki {

template <typename T, int LPR, int G, bool GROUP_MAX>
__global__ __launch_bounds__(256) void score_kernel(
    const typename T::store_t* __restrict__ klo, const typename T::store_t* __restrict__ q,
    const float* __restrict__ P, float* __restrict__ scores, float* __restrict__ qhat_out,
    int Hkv, int S, int S_cap, int d, int rows_per_block) {
  constexpr int EPC = T::EPC;

  __shared__ float s_q[G][kD];
  __shared__ float s_part[G][kRotParts][kD];
  __shared__ float s_qhat[G][kD];

  const int tid = threadIdx.x;
  const int unit = blockIdx.y;
  const int b = unit / Hkv, h = unit % Hkv;
  const int head0 = (b * Hkv + h) * G;  // first query head of the group, flattened over batch

  // Block 0 of a unit rotates all D columns and publishes qhat for the attention stage.
  const int ncols = (blockIdx.x == 0) ? kD : d;
  rotate_query_block<T, G, 256>(q + (size_t)head0 * kD, P + (size_t)h * kD * kD, ncols, s_q, s_part,
                           s_qhat);
  if (blockIdx.x == 0) {
    for (int i = tid; i < G * kD; i += 256) qhat_out[(size_t)head0 * kD + i] = s_qhat[i / kD][i % kD];
  }

  const int lane = tid & 63;
  const int c = lane % LPR;
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
  score_rows<T, LPR, G, 4>(base, row_bytes, cact, qr, row0, row_end,
                           [&](int row, const float (&sc)[G]) {
                             if constexpr (GROUP_MAX) {
                               float m = sc[0];
#pragma unroll
                               for (int g = 1; g < G; ++g) m = fmaxf(m, sc[g]);
                               scores[(size_t)unit * S + row] = m;
                             } else {
#pragma unroll
                               for (int g = 0; g < G; ++g)
                                 scores[(size_t)(head0 + g) * S + row] = sc[g];
                             }
                           });
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
