// Device-side helpers shared by the Loki kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch.h"

namespace loki {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;  // "no row seen yet" sentinel for running maxima (finite on purpose)

// Rows sequence b holds and rows it keeps (clamped, so a bad entry cannot send a kernel out of
// bounds); S_max and k_max are the batch-wide limits every buffer is laid out for.
__device__ __forceinline__ int seq_rows(const Ragged& rg, int b, int S_max) {
  if (rg.seq_lens == nullptr) return S_max;
  return min(max(rg.seq_lens[b], 1), S_max);
}
__device__ __forceinline__ int seq_keep(const Ragged& rg, int b, int k_max, int S_b) {
  const int k = rg.ks != nullptr ? rg.ks[b] : k_max;
  return max(1, min(k, min(k_max, S_b)));
}

// The (sequence, KV head) whose cache rows batch-entry unit `unit` = b * Hkv + h works on.
__device__ __forceinline__ int cache_unit(const Ragged& rg, int unit, int Hkv) {
  return rg.queries <= 1 ? unit : (unit / Hkv / rg.queries) * Hkv + unit % Hkv;
}

// Row index, from the start of a slab, of row s of cache unit (sequence cb, KV head h): the
// contiguous layout, or through the page table (entries clamped, so a bad one cannot leave the
// pool).
__device__ __forceinline__ long long cache_row(const Paging& pg, int cb, int h, int Hkv, int S_cap,
                                               int s) {
  if (pg.table == nullptr) return ((long long)cb * Hkv + h) * S_cap + s;
  int page = pg.table[(long long)cb * pg.pages_per_seq + (s >> pg.lg_rows)];
  page = min(max(page, 0), pg.n_pages - 1);
  return ((((long long)page * Hkv + h) << pg.lg_rows) | (long long)(s & ((1 << pg.lg_rows) - 1)));
}

// Debug builds (-DLOKI_PHASE_TIMING) stamp the 100 MHz wall clock at phase boundaries of the
// fused kernel's blocks so that its time line can be read back; a no-op otherwise.
#ifdef LOKI_PHASE_TIMING
constexpr int kPhaseSlots = 16;
static __device__ unsigned long long g_phase_ts[8192 * kPhaseSlots];  // one copy per source file
#define LOKI_STAMP(i)                                           \
  do {                                                          \
    if (threadIdx.x == 0 && blockIdx.x < 8192)                  \
      loki::g_phase_ts[blockIdx.x * loki::kPhaseSlots + (i)] = wall_clock64(); \
  } while (0)
#else
#define LOKI_STAMP(i) \
  do {                \
  } while (0)
#endif

// ---- storage types: one 16-byte chunk holds EPC elements ---------------------------------
struct F32 {
  using store_t = float;
  static constexpr int kBytes = 4;
  static constexpr int EPC = 4;
  __device__ static inline void unpack(const uint4& r, float (&f)[4]) {
    f[0] = __uint_as_float(r.x);
    f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z);
    f[3] = __uint_as_float(r.w);
  }
  __device__ static inline float load1(const store_t* p) { return *p; }
  __device__ static inline void store1(store_t* p, float x) { *p = x; }
};

struct BF16 {
  using store_t = uint16_t;
  static constexpr int kBytes = 2;
  static constexpr int EPC = 8;
  __device__ static inline void unpack(const uint4& r, float (&f)[8]) {
    f[0] = __uint_as_float(r.x << 16);
    f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16);
    f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16);
    f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16);
    f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  __device__ static inline float load1(const store_t* p) {
    return __uint_as_float(static_cast<uint32_t>(*p) << 16);
  }
  // fp32 -> bf16, round to nearest, ties to even; NaN stays NaN (v_cvt_pk_bf16_f32)
  __device__ static inline uint16_t round(float x) {
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(x));
  }
  // two conversions in one instruction: `lo` lands in bits 15..0, `hi` in bits 31..16
  __device__ static inline uint32_t round2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
  }
  __device__ static inline void store1(store_t* p, float x) { *p = round(x); }
};

__device__ inline uint4 load16(const void* p) { return *reinterpret_cast<const uint4*>(p); }

// ---- cross-lane movement through DPP (no LDS traffic) ----------------------------------
template <int CTRL>
__device__ inline float dpp_mov(float x) {
  return __int_as_float(
      __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}

constexpr int kDppQuadXor1 = 0xB1;       // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141; // lane i <- lane 7-i inside each 8
constexpr int kDppRowMirror = 0x140;     // lane i <- lane 15-i inside each 16

// Sum over each aligned group of LANES consecutive lanes (LANES a power of two); every lane
// of the group receives the total.  All 64 lanes must be active.
template <int LANES>
__device__ inline float group_allreduce_sum(float x) {
  if constexpr (LANES >= 2) x += dpp_mov<kDppQuadXor1>(x);
  if constexpr (LANES >= 4) x += dpp_mov<kDppQuadXor2>(x);
  if constexpr (LANES >= 8) x += dpp_mov<kDppRowHalfMirror>(x);
  if constexpr (LANES >= 16) x += dpp_mov<kDppRowMirror>(x);
  if constexpr (LANES >= 32) x += __shfl_xor(x, 16);
  if constexpr (LANES >= 64) x += __shfl_xor(x, 32);
  return x;
}

// Maximum over each aligned group of LANES consecutive lanes (LANES <= 16), to every lane.
template <int LANES>
__device__ inline float group_allreduce_max(float x) {
  if constexpr (LANES >= 2) x = fmaxf(x, dpp_mov<kDppQuadXor1>(x));
  if constexpr (LANES >= 4) x = fmaxf(x, dpp_mov<kDppQuadXor2>(x));
  if constexpr (LANES >= 8) x = fmaxf(x, dpp_mov<kDppRowHalfMirror>(x));
  if constexpr (LANES >= 16) x = fmaxf(x, dpp_mov<kDppRowMirror>(x));
  return x;
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Order-preserving map float -> uint32 (larger float <=> larger key); -0 is folded onto +0.
__device__ inline uint32_t float_to_key(float a) {
  uint32_t u = __float_as_uint(a);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}


// Inverse of float_to_key (up to the sign of zero).
__device__ inline float key_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

}  // namespace loki
