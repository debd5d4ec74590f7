// Per-head top-k selection (Algorithm 1 line 6 of arXiv 2406.02542) as stand-alone kernels:
// one block per selecting head reads that head's approximate scores and writes the k selected
// positions (ascending) together with their scores, which the attention stage reuses as the
// low-rank part of the exact logits.
//
//   S <= 16384: select_resident_kernel — every thread keeps its keys in registers
//               (select_impl.h), one read of the scores.
//   larger S:   several blocks per head (mb_*_kernel below); beyond 64 chunks of 16384,
//               select_stream_kernel — the scores are streamed four times by one block
//               (histogram of the leading 11 bits; collect the keys of the threshold bin into
//               LDS and resolve the exact threshold among them; count; ordered write), each
//               wave owning a contiguous range so that the ordered write needs no barrier.
#include "select_impl.h"

namespace loki {

constexpr int kSelKPT = 16;

// Second launch bound: 8 waves per SIMD, i.e. at most 64 VGPRs, so that two 1024-thread blocks
// (or four 512-thread blocks) share a CU and overlap each other's barrier and LDS latencies.
template <int THREADS>
__global__ __launch_bounds__(THREADS, 8) void select_resident_kernel(const float* __restrict__ scores,
                                                                  int32_t* __restrict__ sel_idx,
                                                                  float* __restrict__ sel_score,
                                                                  int S_max, int k_max, int per_thread,
                                                                  int heads_per_seq, Ragged rg) {
  __shared__ ResidentSelectSmem<THREADS> sm;
  const int b = (int)blockIdx.x / heads_per_seq;
  const int S = seq_rows(rg, b, S_max), k = seq_keep(rg, b, k_max, S);
  const float* a = scores + (size_t)blockIdx.x * S_max;
  int32_t* out = sel_idx + (size_t)blockIdx.x * k_max;
  float* outs = sel_score + (size_t)blockIdx.x * k_max;
  for (int i = k + (int)threadIdx.x; i < k_max; i += THREADS) out[i] = -1;  // a sequence keeping fewer rows
  LOKI_STAMP(0);
  resident_select_clear<THREADS>(sm);
  __syncthreads();
  block_select_topk_resident<THREADS, kSelKPT>(a, S, k, per_thread, sm,
                                               [&](int rank, int pos, float score) {
                                                 out[rank] = pos;
                                                 outs[rank] = score;
                                               });
}

constexpr int kStreamThreads = 1024;
constexpr int kStreamWaves = kStreamThreads / 64;
constexpr int kStreamMaxCand = kStreamThreads * kSelKPT;  // 16384 keys = 64 KiB of LDS
constexpr int kStreamTile = 256;                          // positions a wave covers per load

union StreamScratch {
  uint32_t cand[kStreamMaxCand];
  SelectSmem<kStreamThreads> generic;  // only used when the threshold bin overflows `cand`
};

template <bool VEC4>
__global__ __launch_bounds__(kStreamThreads) void select_stream_kernel(
    const float* __restrict__ scores, int32_t* __restrict__ sel_idx, float* __restrict__ sel_score,
    int S_max, int k_max, int heads_per_seq, Ragged rg) {
  const int S = seq_rows(rg, (int)blockIdx.x / heads_per_seq, S_max);
  const int k = seq_keep(rg, (int)blockIdx.x / heads_per_seq, k_max, S);
  // loads a lane keeps in flight: a block streams alone on its CU, so the bytes in flight set
  // its bandwidth (16 x 16 B x 1024 threads = 256 KiB); the unaligned variant uses four
  // scalar loads per step and would spill at that depth
  constexpr int kStreamUnroll = VEC4 ? 16 : 4;
  __shared__ ResidentSelectSmem<kStreamThreads> sm;
  __shared__ StreamScratch scratch;
  __shared__ uint32_t s_wcnt[kStreamWaves][2];
  __shared__ uint32_t s_ncand;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* a = scores + (size_t)blockIdx.x * S_max;
  int32_t* out = sel_idx + (size_t)blockIdx.x * k_max;
  float* outs = sel_score + (size_t)blockIdx.x * k_max;
  for (int i = k + tid; i < k_max; i += kStreamThreads) out[i] = -1;  // a sequence keeping fewer rows

  // wave w owns positions [w0, w1), a whole number of tiles
  const int per_wave =
      ((S + kStreamWaves * kStreamTile - 1) / (kStreamWaves * kStreamTile)) * kStreamTile;
  const int w0 = min(S, wave * per_wave), w1 = min(S, w0 + per_wave);

  auto load4 = [&](int pos, float (&f)[4], bool (&ok)[4]) {
    if (VEC4 && (S & 3) == 0) {  // the head's base and pos are 16-byte aligned, pos + 3 < S
      const bool in = pos < w1;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (in) v = *reinterpret_cast<const float4*>(a + pos);
      f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
      ok[0] = ok[1] = ok[2] = ok[3] = in;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        ok[j] = pos + j < w1;
        f[j] = ok[j] ? a[pos + j] : 0.f;
      }
    }
  };

  LOKI_STAMP(0);
  resident_select_clear<kStreamThreads>(sm);
  if (tid == 0) s_ncand = 0u;
  __syncthreads();

  // pass 1: histogram of key bits 31..21
  for (int tile = w0; tile < w1; tile += kStreamTile * kStreamUnroll) {
    float f[kStreamUnroll][4];
    bool ok[kStreamUnroll][4];
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) load4(tile + u * kStreamTile + lane * 4, f[u], ok[u]);
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (ok[u][j]) atomicAdd(&sm.hist[0][float_to_key(f[u][j]) >> 21], 1u);
  }
  __syncthreads();
  resident_find_bin<kStreamThreads>(sm, 0, (uint32_t)k);
  const uint32_t bin1 = sm.out[0][0];
  const uint32_t rem1 = sm.out[0][1];
  LOKI_STAMP(1);

  // pass 2: collect the keys of the threshold bin
  for (int tile = w0; tile < w1; tile += kStreamTile * kStreamUnroll) {
    float f[kStreamUnroll][4];
    bool ok[kStreamUnroll][4];
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) load4(tile + u * kStreamTile + lane * 4, f[u], ok[u]);
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t key = float_to_key(f[u][j]);
        if (ok[u][j] && (key >> 21) == bin1) {
          const uint32_t slot = atomicAdd(&s_ncand, 1u);
          if (slot < (uint32_t)kStreamMaxCand) scratch.cand[slot] = key;
        }
      }
  }
  __syncthreads();
  LOKI_STAMP(2);
  const uint32_t ncand = s_ncand;
  if (ncand > (uint32_t)kStreamMaxCand) {
    // the threshold bin does not fit (e.g. a long run of equal scores): plain digit passes
    __syncthreads();
    block_select_topk<kStreamThreads>(a, S, k, scratch.generic, [&](int rank, int pos) {
      out[rank] = pos;
      outs[rank] = a[pos];
    });
    return;
  }

  // exact threshold among the candidates: they agree on the leading 11 bits, so rank them on
  // the remaining 21, moved to the top of the word
  uint32_t T, need_eq;
  {
    for (int i = tid; i < 2048; i += kStreamThreads) sm.hist[0][i] = 0u;
    int C = ((int)ncand + kStreamThreads - 1) / kStreamThreads;
    C = (C + 3) & ~3;
    uint32_t ck[kSelKPT];
    uint32_t valid_mask = 0;
#pragma unroll
    for (int i = 0; i < kSelKPT; ++i) {
      const uint32_t p = (uint32_t)(tid * C + i);
      const bool v = i < C && p < ncand;
      ck[i] = v ? (scratch.cand[p] << 11) : 0u;
      valid_mask |= (v ? 1u : 0u) << i;
    }
    __syncthreads();
    uint32_t Tp;
    resident_threshold<kStreamThreads, kSelKPT>(ck, valid_mask, rem1, sm, Tp, need_eq);
    T = (bin1 << 21) | (Tp >> 11);
  }
  LOKI_STAMP(3);

  // pass 3: how many selected rows precede each wave's range
  uint32_t cg = 0, ce = 0;
  for (int tile = w0; tile < w1; tile += kStreamTile * kStreamUnroll) {
    float f[kStreamUnroll][4];
    bool ok[kStreamUnroll][4];
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) load4(tile + u * kStreamTile + lane * 4, f[u], ok[u]);
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t key = float_to_key(f[u][j]);
        cg += (ok[u][j] && key > T) ? 1u : 0u;
        ce += (ok[u][j] && key == T) ? 1u : 0u;
      }
  }
  cg = wave_inclusive_scan_u32(cg);
  ce = wave_inclusive_scan_u32(ce);
  if (lane == 63) {
    s_wcnt[wave][0] = cg;
    s_wcnt[wave][1] = ce;
  }
  __syncthreads();
  uint32_t run_g = 0, run_e = 0;
#pragma unroll
  for (int w = 0; w < kStreamWaves; ++w) {
    const uint32_t tg = s_wcnt[w][0], te = s_wcnt[w][1];
    run_g += (w < wave) ? tg : 0u;
    run_e += (w < wave) ? te : 0u;
  }
  LOKI_STAMP(5);

  // pass 4: ordered write; inside a tile, lane l holds positions tile + 4l .. 4l+3
  for (int tile0 = w0; tile0 < w1; tile0 += kStreamTile * kStreamUnroll) {
    float f[kStreamUnroll][4];
    bool ok[kStreamUnroll][4];
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) load4(tile0 + u * kStreamTile + lane * 4, f[u], ok[u]);
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) {
      const int pos = tile0 + u * kStreamTile + lane * 4;
      bool gt[4], eq[4];
      uint32_t mine = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t key = float_to_key(f[u][j]);
        gt[j] = ok[u][j] && key > T;
        eq[j] = ok[u][j] && key == T;
        mine += (gt[j] ? 1u : 0u) + (eq[j] ? 0x10000u : 0u);
      }
      const uint32_t incl = wave_inclusive_scan_u32(mine);  // per tile at most 256 of each kind
      const uint32_t excl = incl - mine;
      uint32_t g_before = run_g + (excl & 0xffffu), e_before = run_e + (excl >> 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (gt[j] || (eq[j] && e_before < need_eq)) {
          const uint32_t rank = g_before + min(e_before, need_eq);
          out[rank] = pos + j;
          outs[rank] = f[u][j];
        }
        g_before += gt[j] ? 1u : 0u;
        e_before += eq[j] ? 1u : 0u;
      }
      const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
      run_g += tot & 0xffffu;
      run_e += tot >> 16;
    }
  }
  LOKI_STAMP(6);
}

// ---- long sequences: several blocks per head ---------------------------------------------------
// One CU cannot stream a long score row fast enough (its outstanding-miss budget caps it at a
// few tens of GB/s), so for S > 16384 a head's scores are cut into chunks of 16384 positions
// and the selection runs as five small kernels:
//   hist     (chunk, head)  11-bit digit histogram of the chunk -> global
//   bin      (head)         sum the chunk histograms, find the threshold bin
//   collect  (chunk, head)  keys of the threshold bin -> per-chunk candidate lists; count of
//                           keys in higher bins
//   resolve  (head)         exact threshold T among the candidates, rank offset of every chunk
//   write    (chunk, head)  ordered emission with those offsets
// If a chunk's candidate list overflows (long runs of equal scores), `resolve` runs the plain
// digit-pass selection for that head by itself and `write` skips it.
constexpr int kMbThreads = 1024;
constexpr int kMbChunk = kMbThreads * kSelKPT;  // 16384 positions per block

__host__ __device__ inline int mb_cand_cap(int nc) { return (kMbChunk / nc) & ~(kSelKPT - 1); }
// per-head words of bookkeeping: cand_cnt[nc], gt_hi[nc], base[nc][2], bin1, rem1, T, need_eq, skip
__host__ __device__ inline int mb_meta_stride(int nc) { return 4 * nc + 8; }

// Streams the n scores at `a` through f(key) with four 16-byte loads per lane in flight.  The
// two counting passes need no key to stay in registers, so when there are enough (chunk, head)
// pairs they run as small blocks, eight to a CU, whose load and LDS phases overlap; a small grid
// keeps 1024-thread blocks so that a CU still has 16 waves.
template <int kMbStreamThreads, typename F>
__device__ __forceinline__ void mb_stream_keys(const float* __restrict__ a, int n, F f) {
  const int tid = threadIdx.x;
  if (n <= 0) return;  // (a negative n would make the tail loop below re-read rows before `a`)
  if ((reinterpret_cast<uintptr_t>(a) & 15u) == 0) {
    const int n4 = n >> 2;  // whole 16-byte words
    const float4* a4 = reinterpret_cast<const float4*>(a);
    int i = tid;
    for (; i + 3 * kMbStreamThreads < n4; i += 4 * kMbStreamThreads) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = a4[i + u * kMbStreamThreads];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        f(float_to_key(v[u].x));
        f(float_to_key(v[u].y));
        f(float_to_key(v[u].z));
        f(float_to_key(v[u].w));
      }
    }
    for (; i < n4; i += kMbStreamThreads) {
      const float4 v = a4[i];
      f(float_to_key(v.x));
      f(float_to_key(v.y));
      f(float_to_key(v.z));
      f(float_to_key(v.w));
    }
    for (int j = 4 * n4 + tid; j < n; j += kMbStreamThreads) f(float_to_key(a[j]));
  } else {
    for (int j = tid; j < n; j += kMbStreamThreads) f(float_to_key(a[j]));
  }
}

template <int kMbStreamThreads>
__global__ __launch_bounds__(kMbStreamThreads) void mb_hist_kernel(const float* __restrict__ scores,
                                                                   uint32_t* __restrict__ hist_part,
                                                                   int S_max, int nc, int heads_per_seq,
                                                                   Ragged rg) {
  __shared__ uint32_t s_hist[2048];
  const int tid = threadIdx.x, chunk = blockIdx.x, head = blockIdx.y;
  const int S = seq_rows(rg, head / heads_per_seq, S_max);
  const int c0 = chunk * kMbChunk, n = max(min(S - c0, kMbChunk), 0);  // 0 past a short sequence's end
  for (int i = tid; i < 2048; i += kMbStreamThreads) s_hist[i] = 0u;
  __syncthreads();
  mb_stream_keys<kMbStreamThreads>(scores + (size_t)head * S_max + c0, n,
                                   [&](uint32_t key) { atomicAdd(&s_hist[key >> 21], 1u); });
  __syncthreads();
  uint32_t* dst = hist_part + ((size_t)head * nc + chunk) * 2048;
  for (int i = tid; i < 2048; i += kMbStreamThreads) dst[i] = s_hist[i];
}

__global__ __launch_bounds__(kMbThreads) void mb_bin_kernel(const uint32_t* __restrict__ hist_part,
                                                            uint32_t* __restrict__ meta,
                                                            int32_t* __restrict__ sel_idx, int S_max,
                                                            int k_max, int nc, int heads_per_seq,
                                                            Ragged rg) {
  __shared__ ResidentSelectSmem<kMbThreads> sm;
  const int tid = threadIdx.x, head = blockIdx.x;
  const int k = seq_keep(rg, head / heads_per_seq, k_max, seq_rows(rg, head / heads_per_seq, S_max));
  for (int i = k + tid; i < k_max; i += kMbThreads)
    sel_idx[(size_t)head * k_max + i] = -1;  // a sequence keeping fewer rows
  const uint32_t* src = hist_part + (size_t)head * nc * 2048;
  uint32_t h0 = 0, h1 = 0;
  for (int c = 0; c < nc; ++c) {
    h0 += src[(size_t)c * 2048 + tid];
    h1 += src[(size_t)c * 2048 + tid + kMbThreads];
  }
  sm.hist[0][tid] = h0;
  sm.hist[0][tid + kMbThreads] = h1;
  __syncthreads();
  resident_find_bin<kMbThreads>(sm, 0, (uint32_t)k);
  if (tid == 0) {
    uint32_t* m = meta + (size_t)head * mb_meta_stride(nc) + 4 * nc;
    m[0] = sm.out[0][0];  // bin1
    m[1] = sm.out[0][1];  // rows still needed from inside bin1
    m[4] = 0u;            // skip flag
  }
}

template <int kMbStreamThreads>
__global__ __launch_bounds__(kMbStreamThreads) void mb_collect_kernel(const float* __restrict__ scores,
                                                                      uint32_t* __restrict__ meta,
                                                                      uint32_t* __restrict__ cand,
                                                                      int S_max, int nc,
                                                                      int heads_per_seq, Ragged rg) {
  __shared__ uint32_t s_ncand, s_gt;
  const int tid = threadIdx.x, lane = tid & 63, chunk = blockIdx.x, head = blockIdx.y;
  const int S = seq_rows(rg, head / heads_per_seq, S_max);
  const int c0 = chunk * kMbChunk, n = max(min(S - c0, kMbChunk), 0);  // 0 past a short sequence's end
  uint32_t* m = meta + (size_t)head * mb_meta_stride(nc);
  const uint32_t bin1 = m[4 * nc];
  const int cap = mb_cand_cap(nc);
  uint32_t* my_cand = cand + (size_t)head * kMbChunk + (size_t)chunk * cap;
  if (tid == 0) {
    s_ncand = 0u;
    s_gt = 0u;
  }
  __syncthreads();
  uint32_t gt = 0;
  mb_stream_keys<kMbStreamThreads>(scores + (size_t)head * S_max + c0, n, [&](uint32_t key) {
    const uint32_t b = key >> 21;
    gt += b > bin1 ? 1u : 0u;
    if (b == bin1) {
      const uint32_t slot = atomicAdd(&s_ncand, 1u);
      if (slot < (uint32_t)cap) my_cand[slot] = key;
    }
  });
  gt = wave_inclusive_scan_u32(gt);
  if (lane == 63) atomicAdd(&s_gt, gt);
  __syncthreads();
  if (tid == 0) {
    m[chunk] = s_ncand;      // may exceed cap: resolve then takes the slow road
    m[nc + chunk] = s_gt;
  }
}

__global__ __launch_bounds__(kMbThreads) void mb_resolve_kernel(
    const float* __restrict__ scores, uint32_t* __restrict__ meta, const uint32_t* __restrict__ cand,
    int32_t* __restrict__ sel_idx, float* __restrict__ sel_score, int S_max, int k_max, int nc,
    int heads_per_seq, Ragged rg) {
  __shared__ ResidentSelectSmem<kMbThreads> sm;
  __shared__ SelectSmem<kMbThreads> generic;
  const int S = seq_rows(rg, (int)blockIdx.x / heads_per_seq, S_max);
  const int k = seq_keep(rg, (int)blockIdx.x / heads_per_seq, k_max, S);
  __shared__ uint32_t s_cg[64], s_ce[64];
  __shared__ uint32_t s_over;
  const int tid = threadIdx.x, head = blockIdx.x;
  uint32_t* m = meta + (size_t)head * mb_meta_stride(nc);
  const int cap = mb_cand_cap(nc);
  if (tid == 0) s_over = 0u;
  resident_select_clear<kMbThreads>(sm);
  if (tid < 64) {
    s_cg[tid] = 0u;
    s_ce[tid] = 0u;
  }
  __syncthreads();
  if (tid < nc && m[tid] > (uint32_t)cap) s_over = 1u;
  __syncthreads();
  if (s_over) {
    if (tid == 0) m[4 * nc + 4] = 1u;
    const float* a = scores + (size_t)head * S_max;
    int32_t* out = sel_idx + (size_t)head * k_max;
    float* outs = sel_score + (size_t)head * k_max;
    block_select_topk<kMbThreads>(a, S, k, generic, [&](int rank, int pos) {
      out[rank] = pos;
      outs[rank] = a[pos];
    });
    return;
  }
  // thread t holds candidate slots [16 t, 16 t + 16), all inside one chunk's list
  const int slot0 = tid * kSelKPT;
  const int ct = slot0 / cap;
  const int ls = slot0 - ct * cap;
  const uint32_t cnt = ct < nc ? m[ct] : 0u;
  const uint32_t* src = cand + (size_t)head * kMbChunk + slot0;
  uint32_t ck[kSelKPT], valid_mask = 0;
#pragma unroll
  for (int i = 0; i < kSelKPT; ++i) {
    const bool v = (uint32_t)(ls + i) < cnt;
    ck[i] = v ? (src[i] << 11) : 0u;   // candidates agree on the top 11 bits: rank on the low 21
    valid_mask |= (v ? 1u : 0u) << i;
  }
  uint32_t Tp, need_eq;
  resident_threshold<kMbThreads, kSelKPT>(ck, valid_mask, m[4 * nc + 1], sm, Tp, need_eq);
  // rows of every chunk that precede it in the output: keys above T and keys equal to T
  uint32_t cg = 0, ce = 0;
#pragma unroll
  for (int i = 0; i < kSelKPT; ++i)
    if ((valid_mask >> i) & 1u) {
      cg += ck[i] > Tp;
      ce += ck[i] == Tp;
    }
  if (cg) atomicAdd(&s_cg[ct], cg);
  if (ce) atomicAdd(&s_ce[ct], ce);
  __syncthreads();
  if (tid == 0) {
    uint32_t g = 0, e = 0;
    for (int c = 0; c < nc; ++c) {
      m[2 * nc + 2 * c] = g;
      m[2 * nc + 2 * c + 1] = e;
      g += m[nc + c] + s_cg[c];
      e += s_ce[c];
    }
    m[4 * nc + 2] = (m[4 * nc] << 21) | (Tp >> 11);
    m[4 * nc + 3] = need_eq;
  }
}

// Ordered emission of a chunk's selected rows.  Each wave owns a contiguous run of the chunk:
// one streaming pass counts the rows above and equal to the threshold in every run, the wave
// totals give every run its first rank, and a second pass writes tile by tile in position
// order.  No key has to stay in registers, so small blocks can be used.  (Keeping a wave's run
// in registers instead, to read it once, measured slower: 28-36 us against 25.6 us on the
// long-context workload.)
template <int THREADS>
__global__ __launch_bounds__(THREADS) void mb_write_kernel(const float* __restrict__ scores,
                                                           const uint32_t* __restrict__ meta,
                                                           int32_t* __restrict__ sel_idx,
                                                           float* __restrict__ sel_score, int S_max,
                                                           int k_max, int nc, int heads_per_seq,
                                                           Ragged rg) {
  constexpr int kWaves = THREADS / 64;
  constexpr int kTile = 256;  // positions a wave covers per load: lane l holds 4 l .. 4 l + 3
  __shared__ uint32_t s_wcnt[kWaves][2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x, head = blockIdx.y;
  const int S = seq_rows(rg, head / heads_per_seq, S_max);
  const uint32_t* m = meta + (size_t)head * mb_meta_stride(nc);
  if (m[4 * nc + 4]) return;  // the head was finished by mb_resolve_kernel (uniform)
  const int c0 = chunk * kMbChunk, n = max(min(S - c0, kMbChunk), 0);
  const float* a = scores + (size_t)head * S_max + c0;
  const bool aligned = (reinterpret_cast<uintptr_t>(a) & 15u) == 0;
  const uint32_t T = m[4 * nc + 2], need_eq = m[4 * nc + 3];
  int32_t* out = sel_idx + (size_t)head * k_max;
  float* outs = sel_score + (size_t)head * k_max;

  const int per_wave = ((n + kWaves * kTile - 1) / (kWaves * kTile)) * kTile;
  const int w0 = min(n, wave * per_wave), w1 = min(n, w0 + per_wave);

  auto load4 = [&](int pos, float (&f)[4], bool (&ok)[4]) {
    if (aligned && pos + 3 < w1) {
      const float4 v = *reinterpret_cast<const float4*>(a + pos);
      f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
      ok[0] = ok[1] = ok[2] = ok[3] = true;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        ok[j] = pos + j < w1;
        f[j] = ok[j] ? a[pos + j] : 0.f;
      }
    }
  };

  uint32_t cg = 0, ce = 0;
  for (int tile = w0; tile < w1; tile += 4 * kTile) {
    float f[4][4];
    bool ok[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) load4(tile + u * kTile + lane * 4, f[u], ok[u]);
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t key = float_to_key(f[u][j]);
        cg += (ok[u][j] && key > T) ? 1u : 0u;
        ce += (ok[u][j] && key == T) ? 1u : 0u;
      }
  }
  cg = wave_inclusive_scan_u32(cg);
  ce = wave_inclusive_scan_u32(ce);
  if (lane == 63) {
    s_wcnt[wave][0] = cg;
    s_wcnt[wave][1] = ce;
  }
  __syncthreads();
  uint32_t run_g = m[2 * nc + 2 * chunk], run_e = m[2 * nc + 2 * chunk + 1];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    run_g += (w < wave) ? s_wcnt[w][0] : 0u;
    run_e += (w < wave) ? s_wcnt[w][1] : 0u;
  }

  for (int tile0 = w0; tile0 < w1; tile0 += 4 * kTile) {
    float f[4][4];
    bool ok[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) load4(tile0 + u * kTile + lane * 4, f[u], ok[u]);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int pos = tile0 + u * kTile + lane * 4;
      bool gt[4], eq[4];
      uint32_t mine = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t key = float_to_key(f[u][j]);
        gt[j] = ok[u][j] && key > T;
        eq[j] = ok[u][j] && key == T;
        mine += (gt[j] ? 1u : 0u) + (eq[j] ? 0x10000u : 0u);
      }
      const uint32_t incl = wave_inclusive_scan_u32(mine);  // per tile at most 256 of each kind
      const uint32_t excl = incl - mine;
      uint32_t g_before = run_g + (excl & 0xffffu), e_before = run_e + (excl >> 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (gt[j] || (eq[j] && e_before < need_eq)) {
          const uint32_t rank = g_before + min(e_before, need_eq);
          out[rank] = c0 + pos + j;
          outs[rank] = f[u][j];
        }
        g_before += gt[j] ? 1u : 0u;
        e_before += eq[j] ? 1u : 0u;
      }
      const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
      run_g += tot & 0xffffu;
      run_e += tot >> 16;
    }
  }
}

// ---- long sequences, one pass over the scores -------------------------------------------------
// When the score kernel has already counted the leading 11 key bits of every score into the
// chunk histograms (one token per sequence), the selection needs one pass over the scores:
//   bin        (head)         sum the chunk histograms, find the threshold bin; from the chunk
//                             histograms alone, how many rows of every chunk lie above the bin
//                             and inside it, i.e. where each chunk's rows go in the lists
//                             (folded into every partition block instead, the search cost 64 MB of
//                             histogram reads per step on the long-context workload and the
//                             stage took twice as long)
//   partition  (chunk, head)  keys in registers: rows above the bin are certain and go to the
//                             index list in position order; rows inside the bin go to the
//                             head's candidate list (key and position), also in position order
//   resolve    (head)         exact threshold among the candidates; the chosen ones are appended
//                             to the index list (if the candidates overflow their list — long
//                             runs of equal scores — the plain digit-pass selection runs instead)
//   merge      (head)         only when the caller wants the list: ascending merge of the two runs
// The attention stage reads the two runs as they are.
constexpr int kMb2Cap = kMbChunk;  // candidates per head
__host__ __device__ inline int mb2_meta_stride(int nc) { return 8 + 2 * nc; }
// per head: [0] bin, [1] rows needed from inside it, [2] certain rows, [3] candidates,
//           [8 + 2c] certain rows before chunk c, [9 + 2c] candidates before chunk c

__global__ __launch_bounds__(kMbThreads) void mb2_bin_kernel(const uint32_t* __restrict__ hist_part,
                                                             uint32_t* __restrict__ meta, int S_max,
                                                             int k_max, int nc, int heads_per_seq,
                                                             Ragged rg) {
  __shared__ ResidentSelectSmem<kMbThreads> sm;
  __shared__ uint32_t s_gt[64], s_eq[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, head = blockIdx.x;
  const int k = seq_keep(rg, head / heads_per_seq, k_max, seq_rows(rg, head / heads_per_seq, S_max));
  const uint32_t* src = hist_part + (size_t)head * nc * 2048;
  uint32_t h0 = 0, h1 = 0;
  for (int c = 0; c < nc; ++c) {
    h0 += src[(size_t)c * 2048 + tid];
    h1 += src[(size_t)c * 2048 + tid + kMbThreads];
  }
  sm.hist[0][tid] = h0;
  sm.hist[0][tid + kMbThreads] = h1;
  __syncthreads();
  resident_find_bin<kMbThreads>(sm, 0, (uint32_t)k);
  const uint32_t bin1 = sm.out[0][0], rem1 = sm.out[0][1];
  for (int c = wave; c < nc; c += kMbThreads / 64) {  // a wave per chunk
    const uint32_t* hp = src + (size_t)c * 2048;
    uint32_t g = 0;
    for (int b = lane; b < 2048; b += 64) g += (uint32_t)b > bin1 ? hp[b] : 0u;
    g = wave_inclusive_scan_u32(g);
    if (lane == 63) {
      s_gt[c] = g;
      s_eq[c] = hp[bin1];
    }
  }
  __syncthreads();
  if (tid == 0) {
    uint32_t* m = meta + (size_t)head * mb2_meta_stride(nc);
    uint32_t g = 0, e = 0;
    for (int c = 0; c < nc; ++c) {
      m[8 + 2 * c] = g;
      m[9 + 2 * c] = e;
      g += s_gt[c];
      e += s_eq[c];
    }
    m[0] = bin1;
    m[1] = rem1;
    m[2] = g;  // = k - rem1
    m[3] = e;
  }
}

__global__ __launch_bounds__(kMbThreads) void mb2_partition_kernel(
    const float* __restrict__ scores, const uint32_t* __restrict__ meta, int32_t* __restrict__ sel_idx,
    float* __restrict__ sel_score, uint32_t* __restrict__ cand_key, int32_t* __restrict__ cand_pos,
    int S_max, int k_max, int nc, int heads_per_seq, Ragged rg) {
  __shared__ uint32_t s_wg[kMbThreads / 64], s_we[kMbThreads / 64];
  const int chunk = blockIdx.x, head = blockIdx.y;
  const int S = seq_rows(rg, head / heads_per_seq, S_max);
  const int c0 = chunk * kMbChunk, n = max(min(S - c0, kMbChunk), 0);  // 0 past a short sequence's end
  const uint32_t* m = meta + (size_t)head * mb2_meta_stride(nc);
  const uint32_t bin1 = m[0], base_g = m[8 + 2 * chunk], base_e = m[9 + 2 * chunk];
  int32_t* out = sel_idx + (size_t)head * k_max;
  float* outs = sel_score + (size_t)head * k_max;
  uint32_t* ck = cand_key + (size_t)head * kMb2Cap;
  int32_t* cp = cand_pos + (size_t)head * kMb2Cap;
  uint32_t key[kSelKPT];
  uint32_t valid_mask;
  resident_load_keys<kSelKPT>(scores + (size_t)head * S_max + c0, n, kSelKPT, key, valid_mask);
  resident_partition<kMbThreads, kSelKPT>(
      key, valid_mask, kSelKPT, bin1, s_wg, s_we,
      [&](int rank, int pos, uint32_t kk) {
        out[base_g + rank] = c0 + pos;
        outs[base_g + rank] = key_to_float(kk);
      },
      [&](int rank, int pos, uint32_t kk) {
        const uint32_t slot = base_e + (uint32_t)rank;
        if (slot < (uint32_t)kMb2Cap) {
          ck[slot] = kk;
          cp[slot] = c0 + pos;
        }
      });
}

__global__ __launch_bounds__(kMbThreads) void mb2_resolve_kernel(
    const float* __restrict__ scores, uint32_t* __restrict__ meta, const uint32_t* __restrict__ cand_key,
    const int32_t* __restrict__ cand_pos, int32_t* __restrict__ sel_idx, float* __restrict__ sel_score,
    int S_max, int k_max, int nc, int heads_per_seq, Ragged rg) {
  __shared__ ResidentSelectSmem<kMbThreads> sm;
  __shared__ SelectSmem<kMbThreads> generic;
  const int tid = threadIdx.x, head = blockIdx.x;
  const int S = seq_rows(rg, head / heads_per_seq, S_max);
  const int k = seq_keep(rg, head / heads_per_seq, k_max, S);
  uint32_t* m = meta + (size_t)head * mb2_meta_stride(nc);
  const uint32_t rem1 = m[1], n_def = m[2], n_cand = m[3];
  int32_t* out = sel_idx + (size_t)head * k_max;
  float* outs = sel_score + (size_t)head * k_max;
  if (n_cand > (uint32_t)kMb2Cap) {  // uniform
    const float* a = scores + (size_t)head * S_max;
    __syncthreads();  // everyone has read the bookkeeping
    if (tid == 0) m[2] = (uint32_t)k;  // the whole list is one ascending run
    block_select_topk<kMbThreads>(a, S, k, generic, [&](int rank, int pos) {
      out[rank] = pos;
      outs[rank] = a[pos];
    });
    return;
  }
  resident_select_clear<kMbThreads>(sm);
  const uint32_t* ck = cand_key + (size_t)head * kMb2Cap;
  const int32_t* cp = cand_pos + (size_t)head * kMb2Cap;
  uint32_t key[kSelKPT];
  uint32_t valid_mask;
  resident_load_keys<kSelKPT>(ck, (int)n_cand, kSelKPT, key, valid_mask);
#pragma unroll
  for (int i = 0; i < kSelKPT; ++i) key[i] <<= 11;  // candidates agree on the top 11 bits: rank on the low 21
  __syncthreads();
  uint32_t Tp, need_eq;
  resident_threshold<kMbThreads, kSelKPT>(key, valid_mask, rem1, sm, Tp, need_eq);
  resident_compact<kMbThreads, kSelKPT>(key, valid_mask, kSelKPT, Tp, need_eq, 0u, 0u, sm.wave[0],
                                        sm.wave[1], [&](int rank, int local, float) {
                                          out[n_def + rank] = cp[local];
                                          outs[n_def + rank] = key_to_float(ck[local]);
                                        });
}

// The caller's copy of a head's list: the certain rows (ascending) and the chosen candidates
// (ascending) merged into one ascending run, padded with -1 for a sequence that keeps fewer
// than k_max rows.
constexpr int kMergeThreads = 1024;
constexpr int kMergeMaxK = 16384;  // list entries the merge holds in LDS (longer lists: from global)
__global__ __launch_bounds__(kMergeThreads) void mb2_merge_kernel(
    const int32_t* __restrict__ sel_idx, const uint32_t* __restrict__ meta,
    int32_t* __restrict__ user_idx, int S_max, int k_max, int nc, int heads_per_seq, Ragged rg) {
  __shared__ int32_t s_list[kMergeMaxK];
  const int head = blockIdx.x;
  const int k = seq_keep(rg, head / heads_per_seq, k_max, seq_rows(rg, head / heads_per_seq, S_max));
  const int n_def = (int)meta[(size_t)head * mb2_meta_stride(nc) + 2];
  const int32_t* glist = sel_idx + (size_t)head * k_max;
  const bool in_lds = k <= kMergeMaxK;
  if (in_lds) {
    for (int i = threadIdx.x; i < k; i += kMergeThreads) s_list[i] = glist[i];
    __syncthreads();
  }
  const int32_t* list = in_lds ? s_list : glist;
  for (int i = threadIdx.x; i < k_max; i += kMergeThreads) {
    if (i >= k) {
      user_idx[(size_t)head * k_max + i] = -1;
      continue;
    }
    const int pos = list[i];
    const bool certain = i < n_def;
    const int32_t* other = certain ? list + n_def : list;
    int lo = 0, hi = certain ? k - n_def : n_def;
    while (lo < hi) {  // entries of the other run below pos
      const int mid = (lo + hi) >> 1;
      if (other[mid] < pos) lo = mid + 1;
      else hi = mid;
    }
    user_idx[(size_t)head * k_max + (certain ? i : i - n_def) + lo] = pos;
  }
}

int select_chunks(int S) { return S > kMbChunk ? (S + kMbChunk - 1) / kMbChunk : 0; }
size_t select_scratch_words(int S, int n_sel_heads) {
  const int nc = select_chunks(S);
  if (nc == 0 || nc > 64) return 0;
  // chunk histograms, then either form's candidate lists and bookkeeping
  return (size_t)n_sel_heads * ((size_t)nc * 2048 + 2 * (size_t)kMbChunk + mb_meta_stride(nc) + mb2_meta_stride(nc));
}

int select_hist_chunks(const Shape& s, int select_mode) {
  const int nc = select_chunks(s.S);
  // Grouped heads that each select for themselves keep the separate counting passes: with G
  // histograms per score block the counting slows the score kernel by more than the saved pass
  // (long-context workload, 4 heads per KV head: 212 us per step against 230 us).
  if (s.G > 1 && select_mode == 0) return 0;
  return (nc == 0 || nc > 64 || s.rg.queries > 1) ? 0 : nc;
}

static hipError_t launch_select_one_pass(const Shape& s, int heads, const float* scores,
                                         int32_t* sel_idx, float* sel_score, uint32_t* scratch,
                                         int32_t* user_idx, hipStream_t st) {
  const int nc = select_chunks(s.S);
  uint32_t* hist_part = scratch;  // filled by the score kernel
  uint32_t* cand_key = hist_part + (size_t)heads * nc * 2048;
  int32_t* cand_pos = reinterpret_cast<int32_t*>(cand_key + (size_t)heads * kMb2Cap);
  uint32_t* meta = reinterpret_cast<uint32_t*>(cand_pos + (size_t)heads * kMb2Cap);
  const int hps = heads / s.B;
  hipLaunchKernelGGL(mb2_bin_kernel, dim3(heads), dim3(kMbThreads), 0, st, hist_part, meta, s.S, s.k, nc,
                     hps, s.rg);
  hipLaunchKernelGGL(mb2_partition_kernel, dim3(nc, heads), dim3(kMbThreads), 0, st, scores, meta, sel_idx,
                     sel_score, cand_key, cand_pos, s.S, s.k, nc, hps, s.rg);
  hipLaunchKernelGGL(mb2_resolve_kernel, dim3(heads), dim3(kMbThreads), 0, st, scores, meta, cand_key,
                     cand_pos, sel_idx, sel_score, s.S, s.k, nc, hps, s.rg);
  if (user_idx != nullptr)
    hipLaunchKernelGGL(mb2_merge_kernel, dim3(heads), dim3(kMergeThreads), 0, st, sel_idx, meta, user_idx, s.S,
                       s.k, nc, hps, s.rg);
  return hipGetLastError();
}

static hipError_t launch_select_multiblock(const Shape& s, int heads, const float* scores,
                                           int32_t* sel_idx, float* sel_score, uint32_t* scratch,
                                           hipStream_t st) {
  const int nc = select_chunks(s.S);
  uint32_t* hist_part = scratch;
  uint32_t* cand = hist_part + (size_t)heads * nc * 2048;
  uint32_t* meta = cand + (size_t)heads * kMbChunk;
  const dim3 wide(nc, heads), narrow(heads), block(kMbThreads);
  const int hps = heads / s.B;  // selecting heads per sequence
  const bool small_blocks = (long long)nc * heads >= 4 * device_cus();
  if (small_blocks)
    hipLaunchKernelGGL(mb_hist_kernel<256>, wide, dim3(256), 0, st, scores, hist_part, s.S, nc, hps, s.rg);
  else
    hipLaunchKernelGGL(mb_hist_kernel<1024>, wide, dim3(1024), 0, st, scores, hist_part, s.S, nc, hps, s.rg);
  hipLaunchKernelGGL(mb_bin_kernel, narrow, block, 0, st, hist_part, meta, sel_idx, s.S, s.k, nc, hps,
                     s.rg);
  if (small_blocks)
    hipLaunchKernelGGL(mb_collect_kernel<256>, wide, dim3(256), 0, st, scores, meta, cand, s.S, nc, hps, s.rg);
  else
    hipLaunchKernelGGL(mb_collect_kernel<1024>, wide, dim3(1024), 0, st, scores, meta, cand, s.S, nc, hps, s.rg);
  hipLaunchKernelGGL(mb_resolve_kernel, narrow, block, 0, st, scores, meta, cand, sel_idx,
                     sel_score, s.S, s.k, nc, hps, s.rg);
  if (small_blocks)
    hipLaunchKernelGGL(mb_write_kernel<256>, wide, dim3(256), 0, st, scores, meta, sel_idx, sel_score,
                       s.S, s.k, nc, hps, s.rg);
  else
    hipLaunchKernelGGL(mb_write_kernel<1024>, wide, dim3(1024), 0, st, scores, meta, sel_idx, sel_score,
                       s.S, s.k, nc, hps, s.rg);
  return hipGetLastError();
}

#ifdef LOKI_PHASE_TIMING
extern "C" int loki_debug_read_select_ts(unsigned long long* host_dst, size_t count) {
  return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(loki::g_phase_ts),
                                  count * sizeof(unsigned long long));
}
#endif

hipError_t launch_select(const Shape& s, int n_sel_heads, const float* scores, int32_t* sel_idx,
                         float* sel_score, uint32_t* scratch, bool one_pass, int32_t* user_idx,
                         hipStream_t st) {
  if (scratch != nullptr && one_pass)
    return launch_select_one_pass(s, n_sel_heads, scores, sel_idx, sel_score, scratch, user_idx, st);
  if (scratch != nullptr && select_scratch_words(s.S, n_sel_heads) != 0)
    return launch_select_multiblock(s, n_sel_heads, scores, sel_idx, sel_score, scratch, st);
  const int hps = n_sel_heads / s.B;  // selecting heads per sequence
  if (s.S <= 512 * kSelKPT) {
    const int per_thread = (((s.S + 511) / 512) + 3) & ~3;
    hipLaunchKernelGGL(select_resident_kernel<512>, dim3(n_sel_heads), dim3(512), 0, st, scores,
                       sel_idx, sel_score, s.S, s.k, per_thread, hps, s.rg);
  } else if (s.S <= 1024 * kSelKPT) {
    const int per_thread = (((s.S + 1023) / 1024) + 3) & ~3;
    hipLaunchKernelGGL(select_resident_kernel<1024>, dim3(n_sel_heads), dim3(1024), 0, st, scores,
                       sel_idx, sel_score, s.S, s.k, per_thread, hps, s.rg);
  } else if (s.S % 4 == 0) {
    hipLaunchKernelGGL(select_stream_kernel<true>, dim3(n_sel_heads), dim3(kStreamThreads), 0, st,
                       scores, sel_idx, sel_score, s.S, s.k, hps, s.rg);
  } else {
    hipLaunchKernelGGL(select_stream_kernel<false>, dim3(n_sel_heads), dim3(kStreamThreads), 0, st,
                       scores, sel_idx, sel_score, s.S, s.k, hps, s.rg);
  }
  return hipGetLastError();
}

}  // namespace loki
