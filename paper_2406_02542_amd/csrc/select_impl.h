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

constexpr int kSelMaxCand = 1024;  // candidates of the threshold bin ranked directly (<= 2048 / 2)

template <int THREADS>
struct SelectSmem {
  static constexpr int kWaves = THREADS / 64;
  uint32_t hist[2048];  // digit histogram; its first kSelMaxCand words later hold the candidates
  uint32_t wave[kWaves];
  uint32_t out[2];
  uint32_t ncand;
  uint32_t cnt[2][kWaves][2];
};

template <int CTRL, int ROW_MASK, bool BOUND_CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xf, BOUND_CTRL);
}

// Inclusive prefix sum over the 64 lanes of a wave, all in DPP: a shift-and-add scan inside
// each row of 16 lanes, then the row totals are carried into the following rows.
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t x) {
  x += dpp_u32<0x111, 0xf, true>(x);   // row_shr:1, zero shifted in
  x += dpp_u32<0x112, 0xf, true>(x);   // row_shr:2
  x += dpp_u32<0x114, 0xf, true>(x);   // row_shr:4
  x += dpp_u32<0x118, 0xf, true>(x);   // row_shr:8
  x += dpp_u32<0x142, 0xa, false>(x);  // row_bcast:15 into rows 1 and 3
  x += dpp_u32<0x143, 0xc, false>(x);  // row_bcast:31 into rows 2 and 3
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

// Same selection for a score array (LDS or global) small enough for every thread to keep its
// keys in registers: C = per_thread <= KPT keys each, C a multiple of 4, THREADS*C >= S
// (nothing at or past S is read).  Two histogram passes (11 + 11 bits) run on the register
// keys, the second one only over the keys of the first pass's threshold bin; the handful of
// keys that still share all 22 leading bits with the threshold are ranked against each other
// directly (a third, 10-bit pass replaces the ranking if there are more than kSelMaxRank of
// them, e.g. many equal scores).  The compaction is one block-wide exclusive scan of
// per-thread counts.  emit(rank, pos, score) is called exactly k times,
// rank in [0, k) ascending with pos.
//
// resident_select_clear() zeroes both histograms; the caller runs it any time before the
// call (with a barrier in between), e.g. ahead of the scoring loop whose closing barrier
// then covers it.
constexpr int kSelMaxRank = 64;

template <int THREADS>
struct ResidentSelectSmem {
  static constexpr int kWaves = THREADS / 64;
  uint32_t hist[2][2048];
  uint32_t wave[2][kWaves];
  uint32_t out[2][2];
  uint32_t ncand;
  uint32_t cand[kSelMaxRank];
};

template <int THREADS>
__device__ __forceinline__ void resident_select_clear(ResidentSelectSmem<THREADS>& sm) {
  for (int i = threadIdx.x; i < 2 * 2048; i += THREADS) (&sm.hist[0][0])[i] = 0u;
  if (threadIdx.x == 0) sm.ncand = 0u;
}

// As find_threshold_bin, on histogram `which` (2048 bins).  One barrier inside, one at the end.
template <int THREADS>
__device__ __forceinline__ void resident_find_bin(ResidentSelectSmem<THREADS>& sm, int which,
                                                  uint32_t rem) {
  constexpr int kWaves = THREADS / 64;
  constexpr int BPT = 2048 / THREADS;
  static_assert(BPT >= 1, "at most 2048 threads");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int top = 2047 - BPT * tid;
  uint32_t cbin[BPT];
  uint32_t c = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) {
    cbin[i] = sm.hist[which][top - i];
    c += cbin[i];
  }
  uint32_t incl = wave_inclusive_scan_u32(c);
  if (lane == 63) sm.wave[which][wave] = incl;
  __syncthreads();
  uint32_t off = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint32_t t = sm.wave[which][w];
    off += (w < wave) ? t : 0u;
  }
  incl += off;
  uint32_t excl = incl - c;
  if (excl < rem && rem <= incl) {
#pragma unroll
    for (int i = 0; i < BPT; ++i) {
      if (excl < rem && rem <= excl + cbin[i]) {
        sm.out[which][0] = (uint32_t)(top - i);
        sm.out[which][1] = rem - excl;
      }
      excl += cbin[i];
    }
  }
  __syncthreads();
}

// Exact threshold of the rem-th largest of the block's register-resident keys: returns the
// key T and how many keys equal to T are needed (need_eq >= 1).  valid_mask bit i says whether
// key[i] takes part.  Both histograms and sm.ncand must be clear on entry (see
// resident_select_clear) and every thread must be past any earlier use of sm.
template <int THREADS, int KPT>
__device__ __forceinline__ void resident_threshold(const uint32_t (&key)[KPT], uint32_t valid_mask,
                                                   uint32_t rem_in, ResidentSelectSmem<THREADS>& sm,
                                                   uint32_t& T, uint32_t& need_eq) {
  const int tid = threadIdx.x;
#define LOKI_SEL_VALID(i) ((valid_mask >> (i)) & 1u)
  // pass 1: bits 31..21 of every key
#pragma unroll
  for (int i = 0; i < KPT; ++i)
    if (LOKI_SEL_VALID(i)) atomicAdd(&sm.hist[0][key[i] >> 21], 1u);
  __syncthreads();
  resident_find_bin<THREADS>(sm, 0, rem_in);
  const uint32_t bin1 = sm.out[0][0];
  LOKI_STAMP(13);

  // pass 2: bits 20..10 of the keys inside the threshold bin
#pragma unroll
  for (int i = 0; i < KPT; ++i)
    if (LOKI_SEL_VALID(i) && (key[i] >> 21) == bin1) atomicAdd(&sm.hist[1][(key[i] >> 10) & 2047u], 1u);
  __syncthreads();
  resident_find_bin<THREADS>(sm, 1, sm.out[0][1]);
  const uint32_t top22 = (bin1 << 11) | sm.out[1][0];
  const uint32_t rem = sm.out[1][1];
  LOKI_STAMP(14);

  // the keys that share all 22 leading bits with the threshold
#pragma unroll
  for (int i = 0; i < KPT; ++i)
    if (LOKI_SEL_VALID(i) && (key[i] >> 10) == top22) {
      const uint32_t slot = atomicAdd(&sm.ncand, 1u);
      if (slot < (uint32_t)kSelMaxRank) sm.cand[slot] = key[i];
    }
  __syncthreads();
  const uint32_t ncand = sm.ncand;
  if (ncand <= (uint32_t)kSelMaxRank) {
    // T is the candidate with (#greater < rem <= #greater + #equal) among the candidates
    if (tid < (int)ncand) {
      const uint32_t ki = sm.cand[tid];
      uint32_t gt = 0, eq = 0;
      for (uint32_t j = 0; j < ncand; ++j) {
        const uint32_t kj = sm.cand[j];
        gt += kj > ki;
        eq += kj == ki;
      }
      if (gt < rem && rem <= gt + eq) {
        sm.out[0][0] = ki;
        sm.out[0][1] = rem - gt;
      }
    }
    __syncthreads();
    T = sm.out[0][0];
    need_eq = sm.out[0][1];
  } else {
    // many keys agree on 22 bits (e.g. equal scores): resolve bits 9..0 with a third pass,
    // reusing histogram 0 (everyone is past its last read: two barriers ago)
    for (int i = tid; i < 2048; i += THREADS) sm.hist[0][i] = 0u;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < KPT; ++i)
      if (LOKI_SEL_VALID(i) && (key[i] >> 10) == top22) atomicAdd(&sm.hist[0][1024u + (key[i] & 1023u)], 1u);
    __syncthreads();
    resident_find_bin<THREADS>(sm, 0, rem);   // bins 1024..2047 hold the 10-bit digit
    T = (top22 << 10) | (sm.out[0][0] - 1024u);
    need_eq = sm.out[0][1];
  }
#undef LOKI_SEL_VALID
}

// The block's positions are laid out wave by wave: wave w owns the 64*C consecutive positions
// from w*64*C in tiles of 256, and inside a tile lane l holds the 4 positions from 4l — one
// coalesced 16-byte load per lane and tile, and a position order (wave, tile, lane, element)
// that the compaction can follow with per-tile DPP scans and a single barrier.
//
// resident_load_keys: reads a[0..n) in that layout; key[4j + e] is position
// resident_pos0(C) + 256 j + e.
__device__ __forceinline__ int resident_pos0(int C) {
  return (int)(threadIdx.x >> 6) * 64 * C + (int)(threadIdx.x & 63) * 4;
}

// The same for an array that already holds keys (16-byte aligned).
template <int KPT>
__device__ __forceinline__ void resident_load_keys(const uint32_t* a, int n, int C, uint32_t (&key)[KPT],
                                                   uint32_t& valid_mask) {
  constexpr int kTiles = KPT / 4;
  const int wbase = resident_pos0(C);
  valid_mask = 0;
#pragma unroll
  for (int j = 0; j < kTiles; ++j) {
    const int i = 4 * j;
    const int p = wbase + 256 * j;
    key[i + 0] = key[i + 1] = key[i + 2] = key[i + 3] = 0u;
    if (i < C) {
      if (p + 3 < n) {
        const uint4 f = *reinterpret_cast<const uint4*>(a + p);
        key[i + 0] = f.x;
        key[i + 1] = f.y;
        key[i + 2] = f.z;
        key[i + 3] = f.w;
        valid_mask |= 0xfu << i;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (p + e < n) {
            key[i + e] = a[p + e];
            valid_mask |= 1u << (i + e);
          }
      }
    }
  }
}

template <int KPT>
__device__ __forceinline__ void resident_load_keys(const float* a, int n, int C, uint32_t (&key)[KPT],
                                                   uint32_t& valid_mask) {
  constexpr int kTiles = KPT / 4;
  const int wbase = resident_pos0(C);
  const bool aligned = (reinterpret_cast<uintptr_t>(a) & 15u) == 0;
  valid_mask = 0;
#pragma unroll
  for (int j = 0; j < kTiles; ++j) {
    const int i = 4 * j;
    const int p = wbase + 256 * j;
    key[i + 0] = key[i + 1] = key[i + 2] = key[i + 3] = 0u;
    if (i < C) {
      if (aligned && p + 3 < n) {
        const float4 f = *reinterpret_cast<const float4*>(a + p);
        key[i + 0] = float_to_key(f.x);
        key[i + 1] = float_to_key(f.y);
        key[i + 2] = float_to_key(f.z);
        key[i + 3] = float_to_key(f.w);
        valid_mask |= 0xfu << i;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (p + e < n) {
            key[i + e] = float_to_key(a[p + e]);
            valid_mask |= 1u << (i + e);
          }
      }
    }
  }
}

// Ordered emission of the keys > T and of the first need_eq keys == T (counted from
// eq_base equal keys already seen at lower positions); ranks start at gt_base +
// min(eq_base, need_eq).  Per tile a DPP exclusive scan over the lanes (greater in the low
// half-word, equal in the high half-word: a wave holds at most 64*KPT <= 65535 keys), then one
// barrier to learn how many selected rows the earlier waves hold.  wave_g / wave_e are two
// LDS arrays of THREADS/64 words that nobody else touches until the next barrier.
// emit(rank, local position, score).
template <int THREADS, int KPT, typename Emit>
__device__ __forceinline__ void resident_compact(const uint32_t (&key)[KPT], uint32_t valid_mask,
                                                 int C, uint32_t T, uint32_t need_eq,
                                                 uint32_t gt_base, uint32_t eq_base,
                                                 uint32_t* wave_g_tot, uint32_t* wave_e_tot,
                                                 Emit emit) {
  constexpr int kWaves = THREADS / 64;
  constexpr int kTiles = KPT / 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wbase = resident_pos0(C);
  uint32_t excl[kTiles];
  uint32_t wave_g = 0, wave_e = 0;
#pragma unroll
  for (int j = 0; j < kTiles; ++j) {
    uint32_t mine = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if ((valid_mask >> (4 * j + e)) & 1u)
        mine += (key[4 * j + e] > T ? 1u : 0u) + (key[4 * j + e] == T ? 0x10000u : 0u);
    const uint32_t incl = wave_inclusive_scan_u32(mine);
    const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    excl[j] = (wave_g + ((incl - mine) & 0xffffu)) | ((wave_e + ((incl - mine) >> 16)) << 16);
    wave_g += tot & 0xffffu;
    wave_e += tot >> 16;
  }
  if (lane == 0) {
    wave_g_tot[wave] = wave_g;
    wave_e_tot[wave] = wave_e;
  }
  __syncthreads();
  uint32_t before_g = gt_base, before_e = eq_base;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint32_t tg = wave_g_tot[w], te = wave_e_tot[w];
    before_g += (w < wave) ? tg : 0u;
    before_e += (w < wave) ? te : 0u;
  }
#pragma unroll
  for (int j = 0; j < kTiles; ++j) {
    uint32_t g_before = before_g + (excl[j] & 0xffffu), e_before = before_e + (excl[j] >> 16);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if ((valid_mask >> (4 * j + e)) & 1u) {
        const uint32_t kk = key[4 * j + e];
        const bool gt = kk > T, eq = kk == T;
        if (gt || (eq && e_before < need_eq))
          emit((int)(g_before + min(e_before, need_eq)), wbase + 256 * j + e, key_to_float(kk));
        g_before += gt;
        e_before += eq;
      }
  }
}

// Ordered split of the register-resident keys by their leading 11 bits against the threshold
// bin: keys in a higher bin are certain to be selected, keys inside the bin are the candidates
// among which the exact threshold lies.  emit_gt(rank, pos) sees every key above the bin with
// its rank among those (ascending with pos) and its key; emit_eq(rank, pos, key) every key inside the bin
// likewise.  Same layout, scans and single barrier as resident_compact.
template <int THREADS, int KPT, typename EmitGt, typename EmitEq>
__device__ __forceinline__ void resident_partition(const uint32_t (&key)[KPT], uint32_t valid_mask,
                                                   int C, uint32_t bin, uint32_t* wave_g_tot,
                                                   uint32_t* wave_e_tot, EmitGt emit_gt,
                                                   EmitEq emit_eq) {
  constexpr int kWaves = THREADS / 64;
  constexpr int kTiles = KPT / 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wbase = resident_pos0(C);
  uint32_t excl[kTiles];
  uint32_t wave_g = 0, wave_e = 0;
#pragma unroll
  for (int j = 0; j < kTiles; ++j) {
    uint32_t mine = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if ((valid_mask >> (4 * j + e)) & 1u) {
        const uint32_t b = key[4 * j + e] >> 21;
        mine += (b > bin ? 1u : 0u) + (b == bin ? 0x10000u : 0u);
      }
    const uint32_t incl = wave_inclusive_scan_u32(mine);
    const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    excl[j] = (wave_g + ((incl - mine) & 0xffffu)) | ((wave_e + ((incl - mine) >> 16)) << 16);
    wave_g += tot & 0xffffu;
    wave_e += tot >> 16;
  }
  if (lane == 0) {
    wave_g_tot[wave] = wave_g;
    wave_e_tot[wave] = wave_e;
  }
  __syncthreads();
  uint32_t before_g = 0, before_e = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint32_t tg = wave_g_tot[w], te = wave_e_tot[w];
    before_g += (w < wave) ? tg : 0u;
    before_e += (w < wave) ? te : 0u;
  }
#pragma unroll
  for (int j = 0; j < kTiles; ++j) {
    uint32_t g_before = before_g + (excl[j] & 0xffffu), e_before = before_e + (excl[j] >> 16);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if ((valid_mask >> (4 * j + e)) & 1u) {
        const uint32_t kk = key[4 * j + e];
        const uint32_t b = kk >> 21;
        if (b > bin) emit_gt((int)g_before, wbase + 256 * j + e, kk);
        if (b == bin) emit_eq((int)e_before, wbase + 256 * j + e, kk);
        g_before += b > bin;
        e_before += b == bin;
      }
  }
}

// ---- keys in LDS, every thread owning C consecutive positions ------------------------------------
// The array is padded by one word per 32 (position r lives at r + r / 32), so that the lanes of a
// wave, whose runs start C words apart, read different banks.  C is a power of two of at most 32,
// so a run never crosses a multiple of 32 and lies in consecutive words.  Thread t owns positions
// [t C, (t + 1) C); ranks follow the thread order, so everything emitted is ascending in position.
// All reads are unconditional (a run past the end of the data is read and masked out): guarded
// reads cost a branch per key.
__device__ __forceinline__ int padded_pos(int r) { return r + (r >> 5); }
__host__ __device__ inline size_t padded_words(size_t n) { return n + (n >> 5) + 33; }

// bit e set: position t C + e is inside the thread's run and below n
__device__ __forceinline__ uint32_t contiguous_valid_mask(int n, int C) {
  const int nv = max(0, min(C, n - (int)threadIdx.x * C));
  return nv >= 32 ? 0xffffffffu : ((1u << nv) - 1u);
}

template <int KPT>
__device__ __forceinline__ void contiguous_load_keys(const uint32_t* s_key, int n, int C,
                                                     uint32_t (&key)[KPT], uint32_t& valid_mask) {
  const uint32_t* run = s_key + padded_pos((int)threadIdx.x * C);
  valid_mask = contiguous_valid_mask(n, C);
#pragma unroll
  for (int e = 0; e < KPT; ++e) {
    const uint32_t x = run[e];  // (inside the array's slack when e >= C)
    key[e] = ((valid_mask >> e) & 1u) ? x : 0u;
  }
}

// One pass over the block's keys: emit_gt(rank, pos) for every key whose leading bits
// (key >> shift) exceed thr, emit_eq(rank, pos, key) for every key whose leading bits equal it,
// ranks counted separately and ascending with pos.  A thread first builds two bit masks over
// its run, the ranks come from one wave scan and one barrier (wave_tot: a word per wave), and the
// emission loops run once per set bit, not once per key.
template <int THREADS, int KPT, typename EmitGt, typename EmitEq>
__device__ __forceinline__ void contiguous_partition(const uint32_t* s_key, int n, int C, int shift,
                                                     uint32_t thr, uint32_t* wave_tot, EmitGt emit_gt,
                                                     EmitEq emit_eq) {
  constexpr int kWaves = THREADS / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r0 = (int)threadIdx.x * C;
  const uint32_t* run = s_key + padded_pos(r0);
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < KPT; ++e) {
    const uint32_t b = run[e] >> shift;
    gt |= (b > thr ? 1u : 0u) << e;
    eq |= (b == thr ? 1u : 0u) << e;
  }
  const uint32_t vm = contiguous_valid_mask(n, C);
  gt &= vm;
  eq &= vm;
  LOKI_STAMP(3);
  const uint32_t mine = (uint32_t)__popc(gt) | ((uint32_t)__popc(eq) << 16);
  const uint32_t incl = wave_inclusive_scan_u32(mine);
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  LOKI_STAMP(5);
  uint32_t before = incl - mine;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) before += (w < wave) ? wave_tot[w] : 0u;
  int g_rank = (int)(before & 0xffffu), e_rank = (int)(before >> 16);
  while (gt) {
    const int e = __ffs((int)gt) - 1;
    gt &= gt - 1;
    emit_gt(g_rank++, r0 + e);
  }
  while (eq) {
    const int e = __ffs((int)eq) - 1;
    eq &= eq - 1;
    emit_eq(e_rank++, r0 + e, run[e]);
  }
}

// Whole selection for S <= THREADS*C: emit(rank, pos, score) is called exactly k times, rank
// in [0, k) ascending with pos.
template <int THREADS, int KPT, typename Emit>
__device__ __forceinline__ void block_select_topk_resident(const float* a, int S, int k,
                                                           int per_thread,
                                                           ResidentSelectSmem<THREADS>& sm,
                                                           Emit emit) {
  uint32_t key[KPT];
  uint32_t valid_mask;
  resident_load_keys<KPT>(a, S, per_thread, key, valid_mask);
  LOKI_STAMP(11);
  uint32_t T, need_eq;
  resident_threshold<THREADS, KPT>(key, valid_mask, (uint32_t)k, sm, T, need_eq);
  LOKI_STAMP(4);
  // sm.wave[0] / sm.wave[1] were last read two or more barriers ago
  resident_compact<THREADS, KPT>(key, valid_mask, per_thread, T, need_eq, 0u, 0u, sm.wave[0],
                                 sm.wave[1], emit);
  LOKI_STAMP(12);
}

}  // namespace loki
