// Several blocks of one launch that work on ONE (batch, KV head) unit together: each scores
// and attends over its own slice of the unit's rows, and the top-k threshold (Algorithm 1 line 6
// of arXiv 2406.02542) is found over all slices by exchanging digit histograms and the few
// threshold-bin candidates through device memory.  Used when a launch has fewer units than the
// chip has compute units, so that one block per unit would leave most of the chip idle.
//
// Exchange rule: what other blocks of the launch read is stored and loaded with device-scope
// relaxed atomics (written through to / served from the level all XCDs share, see
// attend_impl.h), a block arrives at a meeting point only after its own stores have been
// acknowledged, and it reads the others' data only after it has seen all of them arrive.
//
// The blocks of a unit wait for each other, so all of them must be resident at once: the host
// launches at most one block per compute unit, the members of a unit get workgroup ids that the
// dispatcher sends to the same XCD one after the other, and every wait is bounded (a block that
// gives up raises the launch's error word, writes NaN and leaves; nothing spins forever).
#pragma once

#include "select_impl.h"

namespace loki {

constexpr int kClusterRounds = 3;     // histogram exchanges of one launch at most (11 + 11 + 10 bits)

// Device memory of the exchange (all of it inside the caller's workspace).
struct ClusterArgs {
  uint32_t* counters = nullptr;  // [units][kClusterCounterStride]: the blocks' arrival flags (kClusterFlagStride
                                 // words apart), then the count of finished blocks; zero at launch, and
                                 // left zero by the block that merges the unit
  uint32_t* error = nullptr;     // one word: set when a block gave up waiting
  uint32_t* xhist = nullptr;     // [units][kClusterRounds][C][threads] slots: suffix sums of the digit histograms
  size_t xhist_bytes = 0;
  uint32_t* xcand = nullptr;     // [units][candidate capacity] low key bits of the threshold-bin rows
  size_t xcand_bytes = 0;
  float* partial = nullptr;      // [units * G][C][kD + 2] attention partials
  int C = 1;                     // blocks per unit
  int units = 0;                 // units of the launch (the grid is padded)
  uint32_t spin_limit = kClusterSpinLimit;
};

struct ClusterSmem {
  uint32_t bin, rem;
  uint32_t above[kClusterMax], inbin[kClusterMax];
  uint32_t red[2];
  int ok;
};

__device__ __forceinline__ void cluster_store_u32(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t cluster_load_u32(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Meeting point number `meet` (1, 2, ..) of the unit's C blocks.  Every block owns a flag word in
// a memory channel of its own (no read-modify-write, nobody else's polls on its line): it writes
// the meeting's number there once its own stores are acknowledged, and the first C lanes of its
// first wave poll one flag each until all carry that number.  Returns false when the others did
// not arrive within spin_limit polls.  Every thread of the block calls it.
// poisoned (thread 0's value counts): the workspace's error word was set when the launch began —
// an earlier launch on it gave up and left flags behind; the wait then fails at once.
__device__ __forceinline__ bool cluster_arrive_and_wait(uint32_t* flags, int C, int c, uint32_t meet,
                                                        uint32_t spin_limit, bool poisoned, ClusterSmem& cs) {
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this thread's stores are acknowledged
  __syncthreads();
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    if (lane == 0) cluster_store_u32(flags + c * kClusterFlagStride, meet);
    const uint32_t* f = flags + (lane < C ? lane : 0) * kClusterFlagStride;
    bool ok = lane >= C || lane == c || cluster_load_u32(f) >= meet;
    uint32_t spins = 0;
    while (__ballot(!ok) != 0ull && spins < spin_limit) {
      __builtin_amdgcn_s_sleep(1);
      if (!ok) ok = cluster_load_u32(f) >= meet;
      ++spins;
    }
    const bool all = __ballot(!ok) == 0ull;
    if (lane == 0) cs.ok = (all && !poisoned) ? 1 : 0;
  }
  __syncthreads();
  return cs.ok != 0;
}

// 16-byte device-scope accesses to the exchange area (what a device-scope atomic load / store
// compiles to, four words at a time: buffer instructions with the sc1 policy bit).
typedef uint32_t cluster_u32x4 __attribute__((ext_vector_type(4)));
constexpr int kClusterSc1 = 16;  // cache-policy operand: sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t cluster_buffer(const void* base, size_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00027000);
}
__device__ __forceinline__ cluster_u32x4 cluster_load_x4(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(rs, (int)byte_off, 0, kClusterSc1);
}
__device__ __forceinline__ void cluster_store_x4(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off, cluster_u32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, rs, (int)byte_off, 0, kClusterSc1);
}

// One histogram exchange.  hist: this block's 2048-bin digit histogram in LDS (complete and
// visible).  The block publishes the suffix sums of its histogram (bin b: keys in bins >= b),
// meets the others, adds the C arrays up and finds the bin that holds the rem-th largest key of
// the unit: cs.bin, cs.rem (keys still needed from inside that bin) and, per block, the keys
// above the bin (cs.above) and inside it (cs.inbin).  rem >= 1 and the histograms together
// hold at least rem keys.  Returns false when the wait gave up.
// xh / xh_off: the exchange area and the byte offset of this unit's arrays for this round,
// [C][THREADS] slots of kClusterSlotBytes: thread t's slot holds the suffix sums of its own
// bins (ascending) and of the bin above them, so that a reader needs no other thread's slot.
constexpr int kClusterSlotBytes = 32;
template <int THREADS>
__device__ __forceinline__ bool cluster_hist_round(const uint32_t* hist, __amdgpu_buffer_rsrc_t xh,
                                                   uint32_t xh_off, int C, int c, uint32_t* flags,
                                                   uint32_t meet, uint32_t rem, uint32_t spin_limit,
                                                   bool poisoned, uint32_t* wave_tot, ClusterSmem& cs) {
  constexpr int kWaves = THREADS / 64;
  constexpr int BPT = 2048 / THREADS;
  static_assert(BPT == 4, "a slot holds the sums of four bins and of the bin above");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int top = 2047 - BPT * tid;  // thread t owns bins top - 3 .. top
  uint32_t cbin[BPT], mine = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) {
    cbin[i] = hist[top - i];
    mine += cbin[i];
  }
  uint32_t incl = wave_inclusive_scan_u32(mine);
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint32_t t = wave_tot[w];
    incl += (w < wave) ? t : 0u;
  }
  {
    // keys in bins >= top - 3, top - 2, top - 1, top and top + 1
    const uint32_t s0 = incl, s1 = s0 - cbin[3], s2 = s1 - cbin[2], s3 = s2 - cbin[1], s4 = s3 - cbin[0];
    const uint32_t slot = xh_off + (uint32_t)(c * THREADS + tid) * kClusterSlotBytes;
    cluster_store_x4(xh, slot, cluster_u32x4{s0, s1, s2, s3});
    cluster_store_x4(xh, slot + 16, cluster_u32x4{s4, 0u, 0u, 0u});
  }
  if (!cluster_arrive_and_wait(flags, C, c, meet, spin_limit, poisoned, cs)) return false;
  // sc[cc][j]: block cc's suffix sum at bin top - 3 + j (j = 4: the bin above this thread's)
  uint32_t sc[kClusterMax][BPT + 1];
#pragma unroll
  for (int cc = 0; cc < kClusterMax; ++cc) {
    cluster_u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u};
    if (cc < C) {  // (uniform)
      const uint32_t slot = xh_off + (uint32_t)(cc * THREADS + tid) * kClusterSlotBytes;
      a = cluster_load_x4(xh, slot);
      b = cluster_load_x4(xh, slot + 16);
    }
    sc[cc][0] = a[0];
    sc[cc][1] = a[1];
    sc[cc][2] = a[2];
    sc[cc][3] = a[3];
    sc[cc][4] = b[0];
  }
  uint32_t tot[BPT + 1];
#pragma unroll
  for (int j = 0; j <= BPT; ++j) {
    tot[j] = 0;
#pragma unroll
    for (int cc = 0; cc < kClusterMax; ++cc) tot[j] += sc[cc][j];
  }
#pragma unroll
  for (int j = 0; j < BPT; ++j)
    if (tot[j] >= rem && tot[j + 1] < rem) {  // (true for exactly one bin of the block)
      cs.bin = (uint32_t)(top - BPT + 1 + j);
      cs.rem = rem - tot[j + 1];
#pragma unroll
      for (int cc = 0; cc < kClusterMax; ++cc) {
        cs.above[cc] = sc[cc][j + 1];
        cs.inbin[cc] = sc[cc][j] - sc[cc][j + 1];
      }
    }
  __syncthreads();
  return true;
}

// What a block needs to know of a finished round (read right after it, before the next one).
struct ClusterRound {
  uint32_t bin, rem;
  uint32_t own_above, lower_above;  // keys above the bin: in this block, in the blocks before it
  uint32_t own_inbin, lower_inbin, total_inbin;
};
__device__ __forceinline__ ClusterRound cluster_round_result(const ClusterSmem& cs, int C, int c) {
  ClusterRound r;
  r.bin = cs.bin;
  r.rem = cs.rem;
  r.own_above = r.lower_above = r.own_inbin = r.lower_inbin = r.total_inbin = 0;
#pragma unroll
  for (int cc = 0; cc < kClusterMax; ++cc) {
    const uint32_t a = cs.above[cc], b = cs.inbin[cc];
    if (cc < C) {
      r.total_inbin += b;
      if (cc < c) {
        r.lower_above += a;
        r.lower_inbin += b;
      }
      if (cc == c) {
        r.own_above = a;
        r.own_inbin = b;
      }
    }
  }
  return r;
}

// Sum over the block of a per-thread pair of counts (two 16-bit halves, each total below 65536)
// into cs.red[which]; cs.red[which] must be zero on entry.  The caller's next barrier publishes it.
__device__ __forceinline__ void cluster_block_add(uint32_t packed, ClusterSmem& cs, int which) {
  const uint32_t incl = wave_inclusive_scan_u32(packed);
  if ((threadIdx.x & 63) == 63 && incl != 0u) atomicAdd(&cs.red[which], incl);
}

}  // namespace loki
