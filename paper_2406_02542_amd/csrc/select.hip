// Per-head top-k selection (Algorithm 1 line 6 of arXiv 2406.02542) without sorting.
// Scores are mapped to order-preserving 32-bit keys; three histogram passes (11 + 11 + 10
// bits, most significant first) find the exact key T of the k-th largest score and how many
// rows equal to T are still needed; one ordered compaction pass (wave ballot + prefix
// popcount) then emits the positions of all keys > T plus the first `need_eq` keys == T, in
// ascending position order.  Lowest position wins among equal scores.
#include "common.h"
#include "launch.h"

namespace loki {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

__device__ inline uint32_t wave_inclusive_scan(uint32_t x) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(x, o);
    if (lane >= o) x += y;
  }
  return x;
}

// Finds, scanning bins from the highest down, the bin that holds the rem-th largest key.
// hist has nbins (<= 2 * kSelThreads) entries.  Results land in s_out[0] = bin and
// s_out[1] = how many keys are still needed from inside that bin.  Ends with a barrier.
__device__ inline void find_threshold_bin(const uint32_t* hist, int nbins, uint32_t rem,
                                          uint32_t* s_wave, uint32_t* s_out) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b0 = nbins - 1 - 2 * tid, b1 = b0 - 1;
  const uint32_t c0 = b0 >= 0 ? hist[b0] : 0u;
  const uint32_t c1 = b1 >= 0 ? hist[b1] : 0u;
  const uint32_t c = c0 + c1;
  uint32_t incl = wave_inclusive_scan(c);
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  uint32_t off = 0;
  for (int w = 0; w < wave; ++w) off += s_wave[w];
  incl += off;
  const uint32_t excl = incl - c;
  if (excl < rem && rem <= incl) {
    if (excl + c0 >= rem) {
      s_out[0] = (uint32_t)b0;
      s_out[1] = rem - excl;
    } else {
      s_out[0] = (uint32_t)b1;
      s_out[1] = rem - excl - c0;
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ scores,
                                                             int32_t* __restrict__ sel_idx, int S,
                                                             int k) {
  __shared__ uint32_t s_hist[2048];
  __shared__ uint32_t s_wave[kSelWaves];
  __shared__ uint32_t s_out[2];
  __shared__ uint32_t s_cnt[2][kSelWaves][2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* a = scores + (size_t)blockIdx.x * S;
  int32_t* out = sel_idx + (size_t)blockIdx.x * k;

  uint32_t prefix = 0;      // the bits of T fixed so far, right-aligned
  uint32_t rem = (uint32_t)k;
  // pass p looks at `bits` bits below the already fixed `fixed` most significant bits
  const int pass_bits[3] = {11, 11, 10};
  int fixed = 0;
  for (int p = 0; p < 3; ++p) {
    const int bits = pass_bits[p];
    const int nbins = 1 << bits;
    const int shift = 32 - fixed - bits;
    for (int i = tid; i < nbins; i += kSelThreads) s_hist[i] = 0u;
    __syncthreads();
    for (int pos = tid; pos < S; pos += kSelThreads) {
      const uint32_t key = float_to_key(a[pos]);
      const bool match = (fixed == 0) || ((key >> (32 - fixed)) == prefix);
      if (match) atomicAdd(&s_hist[(key >> shift) & (uint32_t)(nbins - 1)], 1u);
    }
    __syncthreads();
    find_threshold_bin(s_hist, nbins, rem, s_wave, s_out);
    prefix = (prefix << bits) | s_out[0];
    rem = s_out[1];
    fixed += bits;
    __syncthreads();
  }
  const uint32_t T = prefix;
  const uint32_t need_eq = rem;  // 1 <= need_eq <= count(key == T)

  // ordered compaction
  uint32_t base_gt = 0, base_eq = 0;
  int buf = 0;
  for (int tile = 0; tile < S; tile += kSelThreads, buf ^= 1) {
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
      s_cnt[buf][wave][0] = __popcll(mgt);
      s_cnt[buf][wave][1] = __popcll(meq);
    }
    __syncthreads();
    uint32_t wgt = 0, weq = 0, tgt = 0, teq = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const uint32_t cg = s_cnt[buf][w][0], ce = s_cnt[buf][w][1];
      if (w < wave) {
        wgt += cg;
        weq += ce;
      }
      tgt += cg;
      teq += ce;
    }
    const uint32_t gt_before = base_gt + wgt + lgt;
    const uint32_t eq_before = base_eq + weq + leq;
    const bool take = gt || (eq && eq_before < need_eq);
    if (take) out[gt_before + min(eq_before, need_eq)] = pos;
    base_gt += tgt;
    base_eq += teq;
  }
}

hipError_t launch_select(const Shape& s, int n_sel_heads, const float* scores, int32_t* sel_idx,
                         hipStream_t st) {
  hipLaunchKernelGGL(select_kernel, dim3(n_sel_heads), dim3(kSelThreads), 0, st, scores, sel_idx,
                     s.S, s.k);
  return hipGetLastError();
}

}  // namespace loki
