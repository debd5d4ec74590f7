// Key rotation into the PCA basis and append into the split cache
// (Algorithm 1 lines 3-4 of arXiv 2406.02542): khat = k P_h, fp32 accumulation, one
// rounding to the storage type, columns [0,d) to the low-rank slab and [d,D) to the residual.
//
// All rows that share a KV head share P_h, whatever their batch index, so a block works on a
// run of (batch, row) items of ONE head with P_h resident in LDS.
#include "common.h"
#include "launch.h"

namespace loki {

constexpr int kRotThreads = 256;
constexpr int kRotTile = 32;          // rows multiplied per step
constexpr int kRotRowsPerThread = 16; // kRotTile / (kRotThreads / kD)

template <typename T>
__global__ __launch_bounds__(kRotThreads) void rotate_kernel(
    const typename T::store_t* __restrict__ k_new, const float* __restrict__ P,
    typename T::store_t* __restrict__ klo, typename T::store_t* __restrict__ khi, int Hkv,
    int S_cap, int d, int pos, int n_new, int n_items, int items_per_block) {
  using ST = typename T::store_t;
  __shared__ float s_P[kD * kD];        // [128][128]
  __shared__ float s_K[kRotTile * kD];  // [kRotTile][128]

  const int tid = threadIdx.x;
  const int h = blockIdx.y;
  const float* Ph = P + (size_t)h * kD * kD;
  for (int i = tid * 4; i < kD * kD; i += kRotThreads * 4)
    *reinterpret_cast<float4*>(s_P + i) = *reinterpret_cast<const float4*>(Ph + i);

  const int j = tid % kD;
  const int rbase = (tid / kD) * kRotRowsPerThread;
  const int item0 = blockIdx.x * items_per_block;
  const int item1 = min(n_items, item0 + items_per_block);

  for (int t0 = item0; t0 < item1; t0 += kRotTile) {
    __syncthreads();  // previous tile fully consumed (and s_P complete on the first trip)
    for (int i = tid; i < kRotTile * kD; i += kRotThreads) {
      const int it = t0 + i / kD;
      float x = 0.f;
      if (it < item1) {
        const int b = it / n_new, r = it % n_new;
        x = T::load1(k_new + ((size_t)(b * Hkv + h) * n_new + r) * kD + (i % kD));
      }
      s_K[i] = x;
    }
    __syncthreads();
    float acc[kRotRowsPerThread];
#pragma unroll
    for (int r = 0; r < kRotRowsPerThread; ++r) acc[r] = 0.f;
    for (int i4 = 0; i4 < kD; i4 += 4) {
      const float p0 = s_P[(i4 + 0) * kD + j], p1 = s_P[(i4 + 1) * kD + j];
      const float p2 = s_P[(i4 + 2) * kD + j], p3 = s_P[(i4 + 3) * kD + j];
#pragma unroll
      for (int r = 0; r < kRotRowsPerThread; ++r) {
        const float4 kv = *reinterpret_cast<const float4*>(s_K + (rbase + r) * kD + i4);
        acc[r] = fmaf(kv.x, p0, acc[r]);
        acc[r] = fmaf(kv.y, p1, acc[r]);
        acc[r] = fmaf(kv.z, p2, acc[r]);
        acc[r] = fmaf(kv.w, p3, acc[r]);
      }
    }
#pragma unroll
    for (int r = 0; r < kRotRowsPerThread; ++r) {
      const int it = t0 + rbase + r;
      if (it < item1) {
        const int b = it / n_new, rr = it % n_new;
        const size_t row = (size_t)(b * Hkv + h) * S_cap + pos + rr;
        if (j < d)
          T::store1(klo + row * d + j, acc[r]);
        else
          T::store1(khi + row * (kD - d) + (j - d), acc[r]);
      }
    }
  }
}

// ---- matrix-core variant for bf16 caches --------------------------------------------------------
// Khat = K P_h over a run of rows is a genuine [n, 128] x [128, 128] contraction.  A wave's
// 16-byte-per-lane load of a 16-row tile of K is directly the A operand of
// v_mfma_f32_16x16x32_bf16 (lane l: row l%16, columns 8*(l/16)..+7 of a 32-column step); the B
// operand is P_h, which is fp32 and enters as three bf16 terms (24 significant bits) so every
// product is exact and only the fp32 accumulation order differs from the vector kernel.  Each
// of the block's four waves owns 32 output columns and keeps its share of P_h in registers
// (4 steps x 2 column blocks x 3 terms); all four read the same K tiles.
typedef __bf16 rot_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float rot_f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kRotMfmaTiles = 2;  // 16-row tiles per loop trip (8 loads in flight per lane)

__global__ __launch_bounds__(kRotThreads) void rotate_mfma_kernel(
    const uint16_t* __restrict__ k_new, const float* __restrict__ P, uint16_t* __restrict__ klo,
    uint16_t* __restrict__ khi, int Hkv, int S_cap, int d, int pos, int n_new, int n_items,
    int items_per_block) {
  __shared__ float s_P[kD * kD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kgrp = lane >> 4, r16 = lane & 15;
  const int h = blockIdx.y;
  const float* Ph = P + (size_t)h * kD * kD;
  for (int i = tid * 4; i < kD * kD; i += kRotThreads * 4)
    *reinterpret_cast<float4*>(s_P + i) = *reinterpret_cast<const float4*>(Ph + i);
  __syncthreads();

  // this wave's columns: 32*wave + 16*nbi + r16
  rot_bf16x8_t bp[4][2][3];
#pragma unroll
  for (int step = 0; step < 4; ++step)
#pragma unroll
    for (int nbi = 0; nbi < 2; ++nbi) {
      uint32_t w[3][4];
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        uint32_t part[3][2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          float rest = s_P[(32 * step + 8 * kgrp + 2 * e2 + e) * kD + 32 * wave + 16 * nbi + r16];
#pragma unroll
          for (int t = 0; t < 3; ++t) {
            const uint16_t hb = BF16::round(rest);
            rest -= __uint_as_float((uint32_t)hb << 16);  // exact in fp32
            part[t][e] = hb;
          }
        }
#pragma unroll
        for (int t = 0; t < 3; ++t) w[t][e2] = part[t][0] | (part[t][1] << 16);
      }
#pragma unroll
      for (int t = 0; t < 3; ++t)
        bp[step][nbi][t] =
            __builtin_bit_cast(rot_bf16x8_t, make_uint4(w[t][0], w[t][1], w[t][2], w[t][3]));
    }

  const int item0 = blockIdx.x * items_per_block;
  const int item1 = min(n_items, item0 + items_per_block);
  for (int t0 = item0; t0 < item1; t0 += 16 * kRotMfmaTiles) {
    uint4 raw[kRotMfmaTiles][4];
#pragma unroll
    for (int u = 0; u < kRotMfmaTiles; ++u) {
      const int it = t0 + 16 * u + r16;
      const bool valid = it < item1;
      const int b = valid ? it / n_new : 0, r = valid ? it % n_new : 0;
      const char* src = reinterpret_cast<const char*>(k_new) +
                        ((size_t)(b * Hkv + h) * n_new + r) * (kD * 2) + (size_t)kgrp * 16;
#pragma unroll
      for (int step = 0; step < 4; ++step)
        raw[u][step] = valid ? load16(src + step * 64) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < kRotMfmaTiles; ++u) {
      // rows this lane will store: items t0 + 16u + 4*kgrp + i
      size_t dst_row[4];
      bool ok[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int it = t0 + 16 * u + 4 * kgrp + i;
        ok[i] = it < item1;
        const int b = ok[i] ? it / n_new : 0, r = ok[i] ? it % n_new : 0;
        dst_row[i] = (size_t)(b * Hkv + h) * S_cap + pos + r;
      }
#pragma unroll
      for (int nbi = 0; nbi < 2; ++nbi) {
        rot_f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 2; t >= 0; --t)  // smallest terms first
#pragma unroll
          for (int step = 0; step < 4; ++step)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(rot_bf16x8_t, raw[u][step]), bp[step][nbi][t], acc, 0, 0, 0);
        const int col = 32 * wave + 16 * nbi + r16;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (ok[i]) {
            if (col < d)
              klo[dst_row[i] * d + col] = BF16::round(acc[i]);
            else
              khi[dst_row[i] * (kD - d) + (col - d)] = BF16::round(acc[i]);
          }
      }
    }
  }
}

hipError_t launch_rotate(const Shape& s, const void* k_new, const float* P, void* klo, void* khi,
                         int pos, int n_new, hipStream_t st) {
  const long long n_items_ll = (long long)s.B * n_new;
  if (n_items_ll > 0x7fffffffLL) return hipErrorInvalidValue;
  const int n_items = (int)n_items_ll;
  int ipb = 512;
  if (n_items < ipb) ipb = ((n_items + kRotTile - 1) / kRotTile) * kRotTile;
  dim3 grid((n_items + ipb - 1) / ipb, s.Hkv);
  const size_t lds = 0;  // LDS is declared statically in the kernels
  if (s.dtype == 1) {
    int ipb_m = 1024;
    if (n_items < ipb_m) ipb_m = ((n_items + 15) / 16) * 16;
    dim3 grid_m((n_items + ipb_m - 1) / ipb_m, s.Hkv);
    hipLaunchKernelGGL(rotate_mfma_kernel, grid_m, dim3(kRotThreads), 0, st,
                       static_cast<const uint16_t*>(k_new), P, static_cast<uint16_t*>(klo),
                       static_cast<uint16_t*>(khi), s.Hkv, s.S_cap, s.d, pos, n_new, n_items, ipb_m);
    return hipGetLastError();
  }
  if (s.dtype == 0) {
    hipLaunchKernelGGL(rotate_kernel<F32>, grid, dim3(kRotThreads), lds, st,
                       static_cast<const float*>(k_new), P, static_cast<float*>(klo),
                       static_cast<float*>(khi), s.Hkv, s.S_cap, s.d, pos, n_new, n_items, ipb);
  } else {
    hipLaunchKernelGGL(rotate_kernel<BF16>, grid, dim3(kRotThreads), lds, st,
                       static_cast<const uint16_t*>(k_new), P, static_cast<uint16_t*>(klo),
                       static_cast<uint16_t*>(khi), s.Hkv, s.S_cap, s.d, pos, n_new, n_items, ipb);
  }
  return hipGetLastError();
}

}  // namespace loki
