// Exact softmax attention over a list of cache rows (Algorithm 1 lines 7-9 of arXiv 2406.02542
// when the list is the selected set; Section 2 Eq. 1 when it is every row), with an online
// softmax in the log2 domain and scale 1/sqrt(D).
//
// One block owns a run of rows of one unit and NH query heads that share those rows.  A row
// of K (logical 128 columns, possibly split between the low-rank slab and the residual slab)
// and the matching row of V are each read by LPRV consecutive lanes with one 16-byte load per
// lane; the K.q dot product is finished with DPP inside the lane group; every lane keeps the
// running output for its EPC columns of V.  Partial (max, sum, output) triples are merged
// across lane groups, waves and finally across blocks (combine_kernel).
#include "common.h"
#include "launch.h"

namespace loki {

constexpr int kAttThreads = 256;
constexpr int kAttWaves = kAttThreads / 64;
constexpr int kRowsInFlight = 4;    // rows per lane group per loop trip
constexpr int kPartialStride = kD + 2;  // o[128], m, l

template <typename T, int NH, bool GATHER>
__global__ __launch_bounds__(kAttThreads) void attend_kernel(
    const void* __restrict__ k_a,   // GATHER: klo [units, S_cap, d]; dense: K [units, S_cap, 128]
    const void* __restrict__ k_b,   // GATHER: khi [units, S_cap, 128-d]; dense: unused
    const void* __restrict__ v,     // [units, S_cap, 128]
    const void* __restrict__ qv,    // GATHER: qhat fp32 [B*Hq, 128]; dense: q storage [B*Hq, 128]
    const int32_t* __restrict__ sel_idx,  // GATHER: [blocks_y, n]
    float* __restrict__ partial,    // [B*Hq, nsplit, 130] when nsplit > 1
    void* __restrict__ out,         // [B*Hq, 128] storage type when nsplit == 1
    int Hq, int Gq, int S_cap, int d, int n, int rows_per_block, int nsplit) {
  using ST = typename T::store_t;
  constexpr int EPC = T::EPC;
  constexpr int LPRV = kD / EPC;           // lanes per row: 16 (bf16) or 32 (fp32)
  constexpr int RPW = 64 / LPRV;           // rows a wave covers per load instruction
  constexpr int R = kRowsInFlight;
  constexpr int ROWS_PER_TRIP = kAttWaves * RPW * R;

  __shared__ int32_t s_idx[GATHER ? kMaxGatherChunk : 1];
  __shared__ float s_m[kAttWaves][NH], s_l[kAttWaves][NH];
  __shared__ float s_o[kAttWaves][NH][kD];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane % LPRV, rg = lane / LPRV;
  const int head0 = blockIdx.y * NH;              // first query head, flattened over batch
  const int bidx = head0 / Hq;
  const int kv_unit = bidx * (Hq / Gq) + (head0 % Hq) / Gq;

  const int r0 = blockIdx.x * rows_per_block;
  const int r1 = min(n, r0 + rows_per_block);

  if constexpr (GATHER) {
    const int32_t* idx = sel_idx + (size_t)blockIdx.y * n;
    for (int i = tid; i < r1 - r0; i += kAttThreads) s_idx[i] = idx[r0 + i];
    __syncthreads();
  }

  // this lane's slice of the NH query vectors
  float qr[NH][EPC];
#pragma unroll
  for (int g = 0; g < NH; ++g) {
    if constexpr (GATHER) {
      const float* qh = static_cast<const float*>(qv) + (size_t)(head0 + g) * kD + c * EPC;
#pragma unroll
      for (int e = 0; e < EPC; ++e) qr[g][e] = qh[e];
    } else {
      const ST* qh = static_cast<const ST*>(qv) + (size_t)(head0 + g) * kD + c * EPC;
#pragma unroll
      for (int e = 0; e < EPC; ++e) qr[g][e] = T::load1(qh + e);
    }
  }

  // where this lane's 16-byte chunk of a K row lives
  const int nlo = GATHER ? d / EPC : LPRV;   // chunks held by k_a
  const bool in_lo = c < nlo;
  const size_t k_row_bytes = in_lo ? (size_t)(GATHER ? d : kD) * T::kBytes
                                   : (size_t)(kD - d) * T::kBytes;
  const char* k_base = in_lo ? static_cast<const char*>(k_a) + (size_t)c * 16
                             : static_cast<const char*>(k_b) + (size_t)(c - nlo) * 16;
  k_base += (size_t)kv_unit * S_cap * k_row_bytes;
  const size_t v_row_bytes = (size_t)kD * T::kBytes;
  const char* v_base = static_cast<const char*>(v) + (size_t)kv_unit * S_cap * v_row_bytes +
                       (size_t)c * 16;

  const float scale = kLog2e * 0.08838834764831845f;  // log2(e) / sqrt(128)

  float m[NH], l[NH], o[NH][EPC];
#pragma unroll
  for (int g = 0; g < NH; ++g) {
    m[g] = kNegBig;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPC; ++e) o[g][e] = 0.f;
  }

  for (int t0 = r0; t0 < r1; t0 += ROWS_PER_TRIP) {
    bool ok[R];
    uint4 kraw[R], vraw[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const int r = t0 + (j * kAttWaves + wave) * RPW + rg;
      ok[j] = r < r1;
      int row = 0;
      if (ok[j]) row = GATHER ? s_idx[r - r0] : r;
      kraw[j] = ok[j] ? load16(k_base + (size_t)row * k_row_bytes) : make_uint4(0, 0, 0, 0);
      vraw[j] = ok[j] ? load16(v_base + (size_t)row * v_row_bytes) : make_uint4(0, 0, 0, 0);
    }
    float logit[NH][R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      float kf[EPC];
      T::unpack(kraw[j], kf);
#pragma unroll
      for (int g = 0; g < NH; ++g) {
        float p = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) p = fmaf(kf[e], qr[g][e], p);
        p = group_allreduce_sum<LPRV>(p);
        logit[g][j] = ok[j] ? p * scale : kNegBig;
      }
    }
    float vf[R][EPC];
#pragma unroll
    for (int j = 0; j < R; ++j) T::unpack(vraw[j], vf[j]);
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      float mn = m[g];
#pragma unroll
      for (int j = 0; j < R; ++j) mn = fmaxf(mn, logit[g][j]);
      const float corr = fast_exp2(m[g] - mn);
      m[g] = mn;
      float pj[R], ps = 0.f;
#pragma unroll
      for (int j = 0; j < R; ++j) {
        pj[j] = ok[j] ? fast_exp2(logit[g][j] - mn) : 0.f;
        ps += pj[j];
      }
      l[g] = fmaf(l[g], corr, ps);
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        float acc = o[g][e] * corr;
#pragma unroll
        for (int j = 0; j < R; ++j) acc = fmaf(pj[j], vf[j][e], acc);
        o[g][e] = acc;
      }
    }
  }

  // merge the RPW lane groups of each wave (they hold disjoint rows, same columns)
#pragma unroll
  for (int off = LPRV; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      const float m2 = __shfl_xor(m[g], off);
      const float l2 = __shfl_xor(l[g], off);
      const float mn = fmaxf(m[g], m2);
      const float a = fast_exp2(m[g] - mn), b2 = fast_exp2(m2 - mn);
      l[g] = l[g] * a + l2 * b2;
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        const float o2 = __shfl_xor(o[g][e], off);
        o[g][e] = o[g][e] * a + o2 * b2;
      }
      m[g] = mn;
    }
  }
  if (rg == 0) {
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      if (c == 0) {
        s_m[wave][g] = m[g];
        s_l[wave][g] = l[g];
      }
#pragma unroll
      for (int e = 0; e < EPC; ++e) s_o[wave][g][c * EPC + e] = o[g][e];
    }
  }
  __syncthreads();

  // merge the waves; thread t owns column t % 128 of heads t / 128, t / 128 + 2, ...
  for (int i = tid; i < NH * kD; i += kAttThreads) {
    const int g = i / kD, col = i % kD;
    float mn = s_m[0][g];
#pragma unroll
    for (int w = 1; w < kAttWaves; ++w) mn = fmaxf(mn, s_m[w][g]);
    float ls = 0.f, os = 0.f;
#pragma unroll
    for (int w = 0; w < kAttWaves; ++w) {
      const float f = fast_exp2(s_m[w][g] - mn);
      ls = fmaf(s_l[w][g], f, ls);
      os = fmaf(s_o[w][g][col], f, os);
    }
    const size_t head = (size_t)(head0 + g);
    if (nsplit == 1) {
      T::store1(static_cast<ST*>(out) + head * kD + col, os / ls);
    } else {
      float* pr = partial + (head * nsplit + blockIdx.x) * kPartialStride;
      pr[col] = os;
      if (col == 0) {
        pr[kD] = mn;
        pr[kD + 1] = ls;
      }
    }
  }
}

// Merges the nsplit partial results of each query head: out = sum_i o_i 2^(m_i - M) / sum_i l_i 2^(m_i - M).
template <typename T>
__global__ __launch_bounds__(kD) void combine_kernel(const float* __restrict__ partial,
                                                     typename T::store_t* __restrict__ out,
                                                     int nsplit) {
  const size_t head = blockIdx.x;
  const int col = threadIdx.x;
  const float* pr = partial + head * nsplit * kPartialStride;
  float mn = kNegBig;
  for (int i = 0; i < nsplit; ++i) mn = fmaxf(mn, pr[i * kPartialStride + kD]);
  float ls = 0.f, os = 0.f;
  for (int i = 0; i < nsplit; ++i) {
    const float f = fast_exp2(pr[i * kPartialStride + kD] - mn);
    ls = fmaf(pr[i * kPartialStride + kD + 1], f, ls);
    os = fmaf(pr[i * kPartialStride + col], f, os);
  }
  T::store1(out + head * kD + col, os / ls);
}

// ---- launchers ------------------------------------------------------------------------
template <typename T, int NH, bool GATHER>
static hipError_t launch_attend_nh(int blocks_y, int nsplit, int rows_per_block, const void* k_a,
                                   const void* k_b, const void* v, const void* qv,
                                   const int32_t* sel_idx, float* partial, void* out, int Hq, int Gq,
                                   int S_cap, int d, int n, hipStream_t st) {
  hipLaunchKernelGGL((attend_kernel<T, NH, GATHER>), dim3(nsplit, blocks_y), dim3(kAttThreads), 0,
                     st, k_a, k_b, v, qv, sel_idx, partial, out, Hq, Gq, S_cap, d, n,
                     rows_per_block, nsplit);
  return hipGetLastError();
}

template <typename T, bool GATHER>
static hipError_t launch_attend_t(int NH, int blocks_y, int nsplit, int rows_per_block,
                                  const void* k_a, const void* k_b, const void* v, const void* qv,
                                  const int32_t* sel_idx, float* partial, void* out, int Hq, int Gq,
                                  int S_cap, int d, int n, hipStream_t st) {
#define LOKI_ATT(NHV)                                                                          \
  return launch_attend_nh<T, NHV, GATHER>(blocks_y, nsplit, rows_per_block, k_a, k_b, v, qv,   \
                                          sel_idx, partial, out, Hq, Gq, S_cap, d, n, st)
  switch (NH) {
    case 1: LOKI_ATT(1);
    case 2: LOKI_ATT(2);
    case 4: LOKI_ATT(4);
    case 8: LOKI_ATT(8);
    default: return hipErrorInvalidValue;
  }
#undef LOKI_ATT
}

static inline int div_up(int a, int b) { return (a + b - 1) / b; }

hipError_t launch_gather(const Shape& s, int select_mode, int nsplit, const float* qhat,
                         const void* klo, const void* khi, const void* v, const int32_t* sel_idx,
                         float* partial, void* out, hipStream_t st) {
  const int NH = (select_mode == 1) ? s.G : 1;
  const int blocks_y = s.B * s.Hq / NH;
  const int rpb = div_up(s.k, nsplit);
  if (rpb > kMaxGatherChunk) return hipErrorInvalidValue;
  if (s.dtype == 0)
    return launch_attend_t<F32, true>(NH, blocks_y, nsplit, rpb, klo, khi, v, qhat, sel_idx, partial,
                                      out, s.Hq, s.G, s.S_cap, s.d, s.k, st);
  return launch_attend_t<BF16, true>(NH, blocks_y, nsplit, rpb, klo, khi, v, qhat, sel_idx, partial,
                                     out, s.Hq, s.G, s.S_cap, s.d, s.k, st);
}

hipError_t launch_dense(const Shape& s, int nsplit, const void* q, const void* k_full,
                        const void* v, float* partial, void* out, hipStream_t st) {
  const int blocks_y = s.B * s.Hkv;
  const int rpb = div_up(s.S, nsplit);
  if (s.dtype == 0)
    return launch_attend_t<F32, false>(s.G, blocks_y, nsplit, rpb, k_full, nullptr, v, q, nullptr,
                                       partial, out, s.Hq, s.G, s.S_cap, kD, s.S, st);
  return launch_attend_t<BF16, false>(s.G, blocks_y, nsplit, rpb, k_full, nullptr, v, q, nullptr,
                                      partial, out, s.Hq, s.G, s.S_cap, kD, s.S, st);
}

hipError_t launch_combine(const Shape& s, int nsplit, const float* partial, void* out,
                          hipStream_t st) {
  if (s.dtype == 0)
    hipLaunchKernelGGL(combine_kernel<F32>, dim3(s.B * s.Hq), dim3(kD), 0, st, partial,
                       static_cast<float*>(out), nsplit);
  else
    hipLaunchKernelGGL(combine_kernel<BF16>, dim3(s.B * s.Hq), dim3(kD), 0, st, partial,
                       static_cast<uint16_t*>(out), nsplit);
  return hipGetLastError();
}

}  // namespace loki
