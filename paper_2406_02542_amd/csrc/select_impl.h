// Block-wide exact top-k selection over a score array (global memory or LDS), shared by the
// stand-alone select kernel and the fused decode kernel.
//
// Scores are mapped to order-preserving 32-bit keys.  Three histogram passes (11 + 11 + 10
// bits, most significant first) find the key T of the k-th largest score and how many rows
// equal to T are still needed; one ordered compaction pass (wave ballot + prefix popcount)
// then emits every position with key > T plus the first `need_eq` positions with key == T,
// in ascending position order.  Lowest position wins among equal scores; no sort anywhere.
#pragma once

#include "common.h"

namespace loki {

template <int THREADS>
struct SelectSmem {
  static constexpr int kWaves = THREADS / 64;
  uint32_t hist[2048];
  uint32_t wave[kWaves];
  uint32_t out[2];
  uint32_t cnt[2][kWaves][2];
};

__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t x) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(x, o);
    if (lane >= o) x += y;
  }
  return x;
}

// Scanning bins from the highest down, finds the bin holding the rem-th largest key and how
// many keys are still needed from inside it: sm.out[0] = bin, sm.out[1] = remainder.
// Thread t owns the BPT consecutive bins ending at nbins-1-BPT*t.  Ends with a barrier.
template <int THREADS>
__device__ __forceinline__ void find_threshold_bin(SelectSmem<THREADS>& sm, int nbins,
                                                   uint32_t rem) {
  constexpr int BPT = 2048 / THREADS > 1 ? 2048 / THREADS : 1;  // bins per thread (nbins <= 2048)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int top = nbins - 1 - BPT * tid;
  uint32_t cbin[BPT];
  uint32_t c = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) {
    const int b = top - i;
    cbin[i] = b >= 0 ? sm.hist[b] : 0u;
    c += cbin[i];
  }
  uint32_t incl = wave_inclusive_scan_u32(c);
  if (lane == 63) sm.wave[wave] = incl;
  __syncthreads();
  uint32_t off = 0;
  for (int w = 0; w < wave; ++w) off += sm.wave[w];
  incl += off;
  uint32_t excl = incl - c;
  if (excl < rem && rem <= incl) {
#pragma unroll
    for (int i = 0; i < BPT; ++i) {
      if (excl < rem && rem <= excl + cbin[i]) {
        sm.out[0] = (uint32_t)(top - i);
        sm.out[1] = rem - excl;
      }
      excl += cbin[i];
    }
  }
  __syncthreads();
}

// a[0..S) must be visible to the whole block on entry.  emit(rank, pos) is called exactly k
// times over the block, rank in [0, k) ascending with pos.
template <int THREADS, typename Emit>
__device__ __forceinline__ void block_select_topk(const float* a, int S, int k,
                                                  SelectSmem<THREADS>& sm, Emit emit) {
  constexpr int kWaves = THREADS / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  uint32_t prefix = 0;  // the bits of T fixed so far, right-aligned
  uint32_t rem = (uint32_t)k;
  int fixed = 0;
#pragma unroll
  for (int p = 0; p < 3; ++p) {
    const int bits = p < 2 ? 11 : 10;
    const int nbins = 1 << bits;
    const int shift = 32 - fixed - bits;
    for (int i = tid; i < nbins; i += THREADS) sm.hist[i] = 0u;
    __syncthreads();
    for (int pos = tid; pos < S; pos += THREADS) {
      const uint32_t key = float_to_key(a[pos]);
      const bool match = (fixed == 0) || ((key >> (32 - fixed)) == prefix);
      if (match) atomicAdd(&sm.hist[(key >> shift) & (uint32_t)(nbins - 1)], 1u);
    }
    __syncthreads();
    find_threshold_bin<THREADS>(sm, nbins, rem);
    prefix = (prefix << bits) | sm.out[0];
    rem = sm.out[1];
    fixed += bits;
    __syncthreads();
  }
  const uint32_t T = prefix;
  const uint32_t need_eq = rem;  // 1 <= need_eq <= count(key == T)

  uint32_t base_gt = 0, base_eq = 0;
  int buf = 0;
  for (int tile = 0; tile < S; tile += THREADS, buf ^= 1) {
    const int pos = tile + tid;
    const bool valid = pos < S;
    const uint32_t key = valid ? float_to_key(a[pos]) : 0u;
    const bool gt = valid && key > T;
    const bool eq = valid && key == T;
    const unsigned long long mgt = __ballot(gt);
    const unsigned long long meq = __ballot(eq);
    const unsigned long long below = (1ull << lane) - 1ull;
    const uint32_t lgt = __popcll(mgt & below), leq = __popcll(meq & below);
    if (lane == 0) {
      sm.cnt[buf][wave][0] = __popcll(mgt);
      sm.cnt[buf][wave][1] = __popcll(meq);
    }
    __syncthreads();
    uint32_t wgt = 0, weq = 0, tgt = 0, teq = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t cg = sm.cnt[buf][w][0], ce = sm.cnt[buf][w][1];
      if (w < wave) {
        wgt += cg;
        weq += ce;
      }
      tgt += cg;
      teq += ce;
    }
    const uint32_t gt_before = base_gt + wgt + lgt;
    const uint32_t eq_before = base_eq + weq + leq;
    if (gt || (eq && eq_before < need_eq)) emit((int)(gt_before + min(eq_before, need_eq)), pos);
    base_gt += tgt;
    base_eq += teq;
  }
}

}  // namespace loki
