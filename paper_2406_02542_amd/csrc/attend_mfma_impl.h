// Attention over a list of cache rows for SEVERAL query heads that share those rows (grouped
// queries; Section 2 Eq. 1 for the dense baseline, Algorithm 1 lines 7-9 of arXiv 2406.02542
// for a selection shared by a KV group), bf16 caches, on the matrix cores.  Device functions
// shared by the stand-alone kernels (attend_mfma.hip) and the single-launch grouped-query
// kernel (fused_gqa.hip).
//
// A wave works on steps of 32 rows:
//   S[row, head] = K[row, :] . q[head, :]      v_mfma_f32_16x16x32_bf16, A = the 16-byte-per-lane
//                                              load of a 16-row tile of K, B = q^T (16 heads)
//   softmax scalars per head                   lane (head, k-group) sees 8 of the 32 rows; the
//                                              step maximum is shared with two cross-row moves
//   O[head, col] += P[head, row] V[row, col]   A = P straight from the accumulator layout of the
//                                              first product (two bf16 terms), B = V^T, which
//                                              needs rows contiguous per lane: V tiles pass
//                                              through LDS (row pitch 264 B, conflict-free
//                                              2-byte column reads)
// The loads of the next step are issued as soon as the current step's keys have gone into the
// first product and its values into LDS, so they are in flight during the softmax and the
// second product.
#pragma once

#include "attend_impl.h"

namespace loki {

typedef __bf16 am_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float am_f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kAmRows = 32;        // rows per wave step
constexpr int kAmPitch = 264;      // bytes per V row in LDS: 256 + 8 keeps column reads conflict-free
constexpr int kAmStageBytes = kAmRows * kAmPitch;  // per wave

// B operand of the first product from an fp32 (rotated) query: head r16's values at `qh`
// (global or LDS), columns 32*step + 8*kgrp .. +7, as QT bf16 terms.  Columns at or past
// `d_limit` and lanes without a head get zeros.
template <int KSTEPS, int QT>
__device__ __forceinline__ void am_query_operands(const float* qh, bool head_ok, int d_limit,
                                                  am_bf16x8_t (&bq)[KSTEPS][QT]) {
  const int kgrp = (threadIdx.x & 63) >> 4;
#pragma unroll
  for (int step = 0; step < KSTEPS; ++step) {
    const int col = 32 * step + 8 * kgrp;
    const bool col_ok = head_ok && col < d_limit;
    uint32_t w[QT][4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      float rest0 = col_ok ? qh[col + 2 * e2] : 0.f, rest1 = col_ok ? qh[col + 2 * e2 + 1] : 0.f;
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        const uint32_t pk = BF16::round2(rest0, rest1);
        rest0 -= __uint_as_float(pk << 16);            // exact in fp32
        rest1 -= __uint_as_float(pk & 0xffff0000u);
        w[t][e2] = pk;
      }
    }
#pragma unroll
    for (int t = 0; t < QT; ++t)
      bq[step][t] = __builtin_bit_cast(am_bf16x8_t, make_uint4(w[t][0], w[t][1], w[t][2], w[t][3]));
  }
}

// Where this lane's 16-byte chunks of a K row and of a V row live: chunk 4*step + kgrp of the
// logical key row (k_a holds the first d_a columns with row pitch d_a, k_b the rest), chunks
// kgrp + 4*step of the value row.
template <int KSTEPS>
struct AmAddr {
  const char* kptr[KSTEPS];
  size_t kpitch[KSTEPS];
  const char* vptr;
};

// LO_ONLY: every chunk comes from k_a (the logits use its columns only).
template <int KSTEPS, bool LO_ONLY>
__device__ __forceinline__ AmAddr<KSTEPS> am_make_addr(const void* k_a, const void* k_b, const void* v,
                                                       size_t addr_unit, int S_cap, int d_a) {
  const int kgrp = (threadIdx.x & 63) >> 4;
  const int nlo = d_a / 8;  // chunks held by k_a
  AmAddr<KSTEPS> ad;
#pragma unroll
  for (int step = 0; step < KSTEPS; ++step) {
    const int c = 4 * step + kgrp;
    const bool in_lo = c < nlo;
    ad.kpitch[step] = (in_lo || LO_ONLY) ? (size_t)d_a * 2 : (size_t)(kD - d_a) * 2;
    const char* base = (in_lo || LO_ONLY) ? static_cast<const char*>(k_a) + (size_t)(in_lo ? c : 0) * 16
                                          : static_cast<const char*>(k_b) + (size_t)(c - nlo) * 16;
    ad.kptr[step] = base + addr_unit * S_cap * ad.kpitch[step];
  }
  ad.vptr = static_cast<const char*>(v) + addr_unit * S_cap * (kD * 2) + (size_t)kgrp * 16;
  return ad;
}

// Running state of one wave: head r16's maximum and sum over this lane's share of the rows,
// and the output accumulators o[cb][i] = column 16*cb + r16 of head 4*kgrp + i.
struct AmState {
  float m_run, l_run;
  am_f32x4_t o[8];
  __device__ __forceinline__ void init() {
    m_run = kNegBig;
    l_run = 0.f;
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) o[cb] = am_f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
};

// List entries r in [r0, r1): cache row = GATHER ? s_idx[r - r0] : r; the block's WAVES waves
// take steps of 32 entries round-robin.  my_v: this wave's kAmStageBytes of LDS.
template <bool GATHER, int KSTEPS, int QT, int WAVES>
__device__ __forceinline__ void am_attend_rows(const AmAddr<KSTEPS>& ad,
                                               const am_bf16x8_t (&bq)[KSTEPS][QT],
                                               const int32_t* s_idx, int r0, int r1,
                                               unsigned char* my_v, AmState& st) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int r16 = lane & 15, kgrp = lane >> 4;
  int base = r0 + wave * kAmRows;
  if (base >= r1) return;

  uint4 kraw[2][KSTEPS], vraw[2][4];
  // two 16-row tiles of K (A operands) and of V (to LDS); rows past the end re-read the last one
  auto issue = [&](int b) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int r = min(b + 16 * t + r16, r1 - 1);
      const int row = GATHER ? s_idx[r - r0] : r;
#pragma unroll
      for (int step = 0; step < 4; ++step) {
        if (step < KSTEPS) kraw[t][step] = load16(ad.kptr[step] + (size_t)row * ad.kpitch[step]);
        vraw[t][step] = load16(ad.vptr + (size_t)row * (kD * 2) + step * 64);
      }
    }
  };
  issue(base);
  for (; base < r1; base += WAVES * kAmRows) {
    // ---- S = K q^T: acc[t][i] = logit of row base + 16 t + 4 kgrp + i for head r16 -----------
    am_f32x4_t s_acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      s_acc[t] = am_f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int qt = QT - 1; qt >= 0; --qt)
#pragma unroll
        for (int step = 0; step < KSTEPS; ++step)
          s_acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              __builtin_bit_cast(am_bf16x8_t, kraw[t][step]), bq[step][qt], s_acc[t], 0, 0, 0);
    }
    // ---- V tiles to LDS, row-major with padded pitch ------------------------------------------
    __builtin_amdgcn_wave_barrier();  // the previous step's column reads are done
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int step = 0; step < 4; ++step)
      {  // the pitch keeps rows 8-byte aligned only: two 8-byte stores per chunk
        unsigned char* dst = my_v + (16 * t + r16) * kAmPitch + (4 * step + kgrp) * 16;
        *reinterpret_cast<uint2*>(dst) = make_uint2(vraw[t][step].x, vraw[t][step].y);
        *reinterpret_cast<uint2*>(dst + 8) = make_uint2(vraw[t][step].z, vraw[t][step].w);
      }
    // ---- the next step's loads, in flight during the softmax and the second product ----------
    issue(base + WAVES * kAmRows);
    // ---- softmax scalars of head r16 -----------------------------------------------------------
    float logit[2][4];
    float smax = kNegBig;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool ok = base + 16 * t + 4 * kgrp + i < r1;
        logit[t][i] = ok ? s_acc[t][i] * kSoftmaxScaleLog2 : kNegBig;
        smax = fmaxf(smax, logit[t][i]);
      }
    smax = fmaxf(smax, __shfl_xor(smax, 16));
    smax = fmaxf(smax, __shfl_xor(smax, 32));
    const float m_new = fmaxf(st.m_run, smax);
    const float corr = fast_exp2(st.m_run - m_new);
    st.m_run = m_new;
    float p[8], psum = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool ok = base + 16 * t + 4 * kgrp + i < r1;
        p[4 * t + i] = ok ? fast_exp2(logit[t][i] - m_new) : 0.f;
        psum += p[4 * t + i];
      }
    st.l_run = fmaf(st.l_run, corr, psum);
    // A operand of the second product: P[head r16][k = 8 kgrp + e], two bf16 terms
    uint32_t ph[4], pl[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      ph[e2] = BF16::round2(p[2 * e2], p[2 * e2 + 1]);
      pl[e2] = BF16::round2(p[2 * e2] - __uint_as_float(ph[e2] << 16),
                            p[2 * e2 + 1] - __uint_as_float(ph[e2] & 0xffff0000u));
    }
    const am_bf16x8_t a_hi = __builtin_bit_cast(am_bf16x8_t, make_uint4(ph[0], ph[1], ph[2], ph[3]));
    const am_bf16x8_t a_lo = __builtin_bit_cast(am_bf16x8_t, make_uint4(pl[0], pl[1], pl[2], pl[3]));
    // ---- rescale the running output when some head's maximum moved ---------------------------
    if (__ballot(corr != 1.0f) != 0ull) {
      float c4[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) c4[i] = __shfl(corr, 4 * kgrp + i);  // lane of head 4 kgrp + i
#pragma unroll
      for (int cb = 0; cb < 8; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i) st.o[cb][i] *= c4[i];
    }
    // ---- O += P V: B operand = V^T, rows (k index 8 kgrp + e) -> tile e/4, row 4 kgrp + e%4 ----
    __builtin_amdgcn_wave_barrier();  // the V tiles above are written
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
      uint32_t w[4];
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const int e = 2 * e2;
        const int rl0 = 16 * (e / 4) + 4 * kgrp + (e % 4);
        const uint32_t x0 = *reinterpret_cast<const uint16_t*>(my_v + rl0 * kAmPitch + (16 * cb + r16) * 2);
        const uint32_t x1 = *reinterpret_cast<const uint16_t*>(my_v + (rl0 + 1) * kAmPitch + (16 * cb + r16) * 2);
        w[e2] = x0 | (x1 << 16);
      }
      const am_bf16x8_t bv = __builtin_bit_cast(am_bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
      st.o[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo, bv, st.o[cb], 0, 0, 0);
      st.o[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi, bv, st.o[cb], 0, 0, 0);
    }
  }
}

// Wave totals (sum over the four k-groups) into LDS, one (m, l, o[128]) per wave and head.
// Ends with a barrier.
template <int NH, int WAVES>
__device__ __forceinline__ void am_publish(AmState& st, MergeSmem<WAVES, NH>& sm) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, kgrp = lane >> 4;
  st.l_run += __shfl_xor(st.l_run, 16);
  st.l_run += __shfl_xor(st.l_run, 32);
  if (kgrp == 0 && r16 < NH) {
    sm.m[wave][r16] = st.m_run;
    sm.l[wave][r16] = st.l_run;
  }
#pragma unroll
  for (int cb = 0; cb < 8; ++cb)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int head = 4 * kgrp + i;
      if (head < NH) sm.o[wave][head][16 * cb + r16] = st.o[cb][i];
    }
  __syncthreads();
}

}  // namespace loki
