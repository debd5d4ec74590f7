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

hipError_t launch_rotate(const Shape& s, const void* k_new, const float* P, void* klo, void* khi,
                         int pos, int n_new, hipStream_t st) {
  const long long n_items_ll = (long long)s.B * n_new;
  if (n_items_ll > 0x7fffffffLL) return hipErrorInvalidValue;
  const int n_items = (int)n_items_ll;
  int ipb = 512;
  if (n_items < ipb) ipb = ((n_items + kRotTile - 1) / kRotTile) * kRotTile;
  dim3 grid((n_items + ipb - 1) / ipb, s.Hkv);
  const size_t lds = 0;  // LDS is declared statically in the kernel (80 KiB of the CU's 160 KiB)
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
