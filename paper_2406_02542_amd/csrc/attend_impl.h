// Exact softmax attention over a list of cache rows with an online softmax in the log2
// domain and scale 1/sqrt(D) (Algorithm 1 lines 7-9 of arXiv 2406.02542 for the selected set,
// Section 2 Eq. 1 for every row).  Shared by the stand-alone attention kernels and the fused
// decode kernel.
//
// A row of K (128 logical columns, possibly split between the low-rank slab and the residual
// slab) and the matching row of V are each read by LPRV consecutive lanes with one 16-byte
// load per lane; the K.q dot product is finished with DPP inside the lane group; every lane
// keeps the running output for its EPC columns of V.
//
// REUSE_LO: the low-rank part of the exact logit, sum_{j<d} qhat_j Khat[s,j], is exactly the
// approximate score the ranking stage already computed, so the lanes that would read the
// low-rank slab read nothing and the saved score is added instead.
#pragma once

#include "common.h"

namespace loki {

#ifndef LOKI_ROWS_IN_FLIGHT
#define LOKI_ROWS_IN_FLIGHT 4
#endif
constexpr int kRowsInFlight = LOKI_ROWS_IN_FLIGHT;  // rows per lane group per loop trip
constexpr int kPartialStride = kD + 2;  // o[128], m, l
constexpr float kSoftmaxScaleLog2 = kLog2e * 0.08838834764831845f;  // log2(e) / sqrt(128)

template <typename T, int NH>
struct AttendAcc {
  float m[NH], l[NH], o[NH][T::EPC];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      m[g] = kNegBig;
      l[g] = 0.f;
#pragma unroll
      for (int e = 0; e < T::EPC; ++e) o[g][e] = 0.f;
    }
  }
};

struct RowAddr {
  const char* k_base;   // this lane's 16-byte chunk of K row 0 of the unit
  size_t k_row_bytes;
  const char* v_base;   // this lane's 16-byte chunk of V row 0 of the unit
  size_t v_row_bytes;
  bool k_load;          // false: this lane's K chunk is covered by the reused score
};

// c = lane's chunk index inside a row (0 .. 128/EPC-1).  k_a holds the first d columns
// (d = 128: the whole row), k_b the rest.  LO_ONLY: the logit uses the first d columns only
// (Algorithm 2, PCAAttn); lanes past them read no key at all.
template <typename T, bool REUSE_LO, bool LO_ONLY = false>
__device__ __forceinline__ RowAddr make_row_addr(const void* k_a, const void* k_b, const void* v,
                                                 size_t kv_unit, int S_cap, int d, int c) {
  const int nlo = d / T::EPC;
  const bool in_lo = c < nlo;
  RowAddr ra;
  ra.k_load = LO_ONLY ? in_lo : !(REUSE_LO && in_lo);
  ra.k_row_bytes = (in_lo || LO_ONLY) ? (size_t)d * T::kBytes : (size_t)(kD - d) * T::kBytes;
  const char* kb = (in_lo || LO_ONLY) ? static_cast<const char*>(k_a) + (size_t)(in_lo ? c : 0) * 16
                                      : static_cast<const char*>(k_b) + (size_t)(c - nlo) * 16;
  ra.k_base = kb + kv_unit * S_cap * ra.k_row_bytes;
  ra.v_row_bytes = (size_t)kD * T::kBytes;
  ra.v_base = static_cast<const char*>(v) + kv_unit * S_cap * ra.v_row_bytes + (size_t)c * 16;
  return ra;
}

// Processes list entries r in [r0, r1): cache row = GATHER ? s_idx[r - r0] : r.  NGROUPS lane
// groups of the block share the entries round-robin; `gid` is this lane's group.
template <typename T, int NH, int NGROUPS, bool GATHER, bool REUSE_LO>
__device__ __forceinline__ void attend_rows(AttendAcc<T, NH>& acc, const float (&qr)[NH][T::EPC],
                                            const RowAddr& ra, const int32_t* s_idx,
                                            const float* s_a, int gid, int r0, int r1) {
  constexpr int EPC = T::EPC;
  constexpr int LPRV = kD / EPC;
  constexpr int R = kRowsInFlight;
  static_assert(!REUSE_LO || NH == 1, "score reuse needs one query head per selection");
  for (int t0 = r0; t0 < r1; t0 += NGROUPS * R) {
    bool ok[R];
    uint4 kraw[R], vraw[R];
    float alo[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const int r = t0 + j * NGROUPS + gid;
      ok[j] = r < r1;
      int row = 0;
      alo[j] = 0.f;
      if (ok[j]) {
        row = GATHER ? s_idx[r - r0] : r;
        if constexpr (REUSE_LO) alo[j] = s_a[r - r0];
      }
      kraw[j] = (ok[j] && ra.k_load) ? load16(ra.k_base + (size_t)row * ra.k_row_bytes)
                                     : make_uint4(0, 0, 0, 0);
      vraw[j] = ok[j] ? load16(ra.v_base + (size_t)row * ra.v_row_bytes) : make_uint4(0, 0, 0, 0);
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
        if constexpr (REUSE_LO) p += alo[j];
        logit[g][j] = ok[j] ? p * kSoftmaxScaleLog2 : kNegBig;
      }
    }
    float vf[R][EPC];
#pragma unroll
    for (int j = 0; j < R; ++j) T::unpack(vraw[j], vf[j]);
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      float mn = acc.m[g];
#pragma unroll
      for (int j = 0; j < R; ++j) mn = fmaxf(mn, logit[g][j]);
      const float corr = fast_exp2(acc.m[g] - mn);
      acc.m[g] = mn;
      float pj[R], ps = 0.f;
#pragma unroll
      for (int j = 0; j < R; ++j) {
        pj[j] = ok[j] ? fast_exp2(logit[g][j] - mn) : 0.f;
        ps += pj[j];
      }
      acc.l[g] = fmaf(acc.l[g], corr, ps);
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        float a = acc.o[g][e] * corr;
#pragma unroll
        for (int j = 0; j < R; ++j) a = fmaf(pj[j], vf[j][e], a);
        acc.o[g][e] = a;
      }
    }
  }
}

template <int WAVES, int NH>
struct MergeSmem {
  float m[WAVES][NH], l[WAVES][NH];
  float o[WAVES][NH][kD];
};

// Merges the lane groups of each wave in registers, then publishes one (m, l, o[128]) per
// wave and head in LDS.  Ends with a barrier.
template <typename T, int NH, int WAVES>
__device__ __forceinline__ void attend_publish(AttendAcc<T, NH>& acc, MergeSmem<WAVES, NH>& sm) {
  constexpr int EPC = T::EPC;
  constexpr int LPRV = kD / EPC;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane % LPRV, rg = lane / LPRV;
#pragma unroll
  for (int off = LPRV; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      const float m2 = __shfl_xor(acc.m[g], off);
      const float l2 = __shfl_xor(acc.l[g], off);
      const float mn = fmaxf(acc.m[g], m2);
      const float a = fast_exp2(acc.m[g] - mn), b2 = fast_exp2(m2 - mn);
      acc.l[g] = acc.l[g] * a + l2 * b2;
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        const float o2 = __shfl_xor(acc.o[g][e], off);
        acc.o[g][e] = acc.o[g][e] * a + o2 * b2;
      }
      acc.m[g] = mn;
    }
  }
  if (rg == 0) {
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      if (c == 0) {
        sm.m[wave][g] = acc.m[g];
        sm.l[wave][g] = acc.l[g];
      }
#pragma unroll
      for (int e = 0; e < EPC; ++e) sm.o[wave][g][c * EPC + e] = acc.o[g][e];
    }
  }
  __syncthreads();
}

// Partial results that another block of the same launch will read (the merge by the last
// block, below) are stored and loaded as device-scope relaxed atomics: such a store is written
// through to the level all XCDs share and such a load is served from there, so no block has to
// write back or invalidate a whole L2 (a device-scope fence per block costs tens of
// microseconds on this part: measured 33 -> 144 us on a 512-block gather).
__device__ __forceinline__ void store_shared_f32(float* p, float v, bool device_scope) {
  if (device_scope) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}
template <bool DEVICE_SCOPE>
__device__ __forceinline__ float load_shared_f32(const float* p) {
  if constexpr (DEVICE_SCOPE) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return *p;
}

// Merge of the nsplit partial results of one query head, column col:
// sum_i o_i 2^(m_i - M) / sum_i l_i 2^(m_i - M).  Loads are issued in independent batches of 8
// splits so that the merge costs a few memory round trips, not one per split.
template <bool DEVICE_SCOPE>
__device__ __forceinline__ float combine_splits(const float* pr, int nsplit, int col) {
  constexpr int B8 = 8;
  float mn = kNegBig;
  for (int i0 = 0; i0 < nsplit; i0 += B8) {
    float mi[B8];
#pragma unroll
    for (int u = 0; u < B8; ++u)
      mi[u] = (i0 + u < nsplit) ? load_shared_f32<DEVICE_SCOPE>(pr + (i0 + u) * kPartialStride + kD) : kNegBig;
#pragma unroll
    for (int u = 0; u < B8; ++u) mn = fmaxf(mn, mi[u]);
  }
  float ls = 0.f, os = 0.f;
  for (int i0 = 0; i0 < nsplit; i0 += B8) {
    float mi[B8], li[B8], oi[B8];
#pragma unroll
    for (int u = 0; u < B8; ++u) {
      const bool ok = i0 + u < nsplit;
      const float* p = pr + (ok ? (i0 + u) : 0) * kPartialStride;
      const float m_ = load_shared_f32<DEVICE_SCOPE>(p + kD), l_ = load_shared_f32<DEVICE_SCOPE>(p + kD + 1);
      const float o_ = load_shared_f32<DEVICE_SCOPE>(p + col);
      mi[u] = ok ? m_ : kNegBig;
      li[u] = ok ? l_ : 0.f;
      oi[u] = ok ? o_ : 0.f;
    }
#pragma unroll
    for (int u = 0; u < B8; ++u) {
      const float f = fast_exp2(mi[u] - mn);
      ls = fmaf(li[u], f, ls);
      os = fmaf(oi[u], f, os);
    }
  }
  return os / ls;
}

// The row splits of a head group are merged by whichever of its blocks finishes last, so the
// merge needs no launch of its own.  Call after the block's partials are stored (with
// store_shared_f32 at device scope), by every thread of the block; `ticket` counts the group's
// finished blocks and is zero when the launch starts.  Every thread waits until its own stores
// are acknowledged (vmcnt(0)), the barrier collects the block, and only then one thread takes
// the ticket with a device-scope atomic; the block that draws the last one reads the others'
// partials with device-scope loads issued after that atomic has returned.  No block waits for
// another.
__device__ __forceinline__ bool splits_all_done(int32_t* ticket, int nsplit) {
  __shared__ int s_last_block;
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0); expcnt and lgkmcnt left alone
  __syncthreads();
  if (threadIdx.x == 0) s_last_block = (atomicAdd(ticket, 1) == nsplit - 1) ? 1 : 0;
  __syncthreads();
  return s_last_block != 0;
}

// Merged (max, sum, output) of head g, column col over the block's waves.
template <int WAVES, int NH>
__device__ __forceinline__ void attend_merged(const MergeSmem<WAVES, NH>& sm, int g, int col,
                                              float& mn, float& ls, float& os) {
  mn = sm.m[0][g];
#pragma unroll
  for (int w = 1; w < WAVES; ++w) mn = fmaxf(mn, sm.m[w][g]);
  ls = 0.f;
  os = 0.f;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) {
    const float f = fast_exp2(sm.m[w][g] - mn);
    ls = fmaf(sm.l[w][g], f, ls);
    os = fmaf(sm.o[w][g][col], f, os);
  }
}

}  // namespace loki
