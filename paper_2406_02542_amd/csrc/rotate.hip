// Key rotation into the PCA basis and append into the split cache
// (Algorithm 1 lines 3-4 of arXiv 2406.02542): khat = k P_h, fp32 accumulation, one
// rounding to the storage type, columns [0,d) to the low-rank slab and [d,D) to the residual.
//
// All rows that share a KV head share P_h, whatever their batch index, so a block works on a
// run of (batch, row) items of ONE head with P_h resident in LDS.
#include <type_traits>

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
    int S_cap, int d, int pos, int n_new, int n_items, int items_per_block, Paging pg) {
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
        const size_t row = (size_t)cache_row(pg, b, h, Hkv, S_cap, pos + rr);
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
// v_mfma_f32_16x16x32_bf16 (lane l: row l%16, columns 8*(l/16)..+7 of a 32-column step).  The B
// operand is P_h, which is fp32: it is split once per block into three bf16 terms (24
// significant bits, so every product is exact and only the fp32 accumulation order differs
// from the vector kernel) and parked in LDS already in operand layout, 96 KiB.  Every wave
// owns whole 16-row tiles (each key row is read from HBM once), prefetches its next tile while
// the 96 matrix instructions of the current one run, packs pairs of neighbouring columns into
// a staging tile in LDS, and writes whole rows from there.
typedef __bf16 rot_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float rot_f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kRotMfmaThreads = 512;
constexpr int kRotMfmaWaves = kRotMfmaThreads / 64;
constexpr int kRotMfmaMinItems = 1024;  // rows per block, at least and at most
constexpr int kRotMfmaMaxItems = 8192;
constexpr int kRotMfmaTPW = 2;        // tiles a wave multiplies per operand fetch
constexpr int kRotTerms = 3;          // bf16 terms P enters with (3: every product exact)

// PAGED: the output rows go through the page table (a separate instantiation, so that the
// contiguous kernel's store addresses stay plain arithmetic).
template <bool PAGED>
__global__ __launch_bounds__(kRotMfmaThreads) void rotate_mfma_kernel(
    const uint16_t* __restrict__ k_new, const float* __restrict__ P, uint16_t* __restrict__ klo,
    uint16_t* __restrict__ khi, int Hkv, int S_cap, int d, int pos, int n_new, int n_items,
    int items_per_block, Paging pg) {
  __shared__ uint4 s_B[kRotTerms][4][8][64];  // [term][32-column step of K][16-column block of Khat][lane]
  // per wave: the rotated tiles of a trip, bf16, before they leave as whole rows (with three
  // terms the two arrays fill the 160 KiB of a CU exactly)
  __shared__ uint4 s_stage[kRotMfmaWaves][kRotMfmaTPW * 16 * 16];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: row bases stay scalar
  const int kgrp = lane >> 4, r16 = lane & 15;
  const int h = blockIdx.y;
  const float* Ph = P + (size_t)h * kD * kD;

  // element P[i][col] belongs to operand (step i/32, block col/16), lane ((i%32)/8)*16 + col%16,
  // slot i%8
  constexpr int kPrep = kD * kD / kRotMfmaThreads;  // 32 elements per thread, all loads in flight
  float pv[kPrep];
#pragma unroll
  for (int n = 0; n < kPrep; ++n) pv[n] = Ph[tid + n * kRotMfmaThreads];
#pragma unroll
  for (int n = 0; n < kPrep; ++n) {
    const int idx = tid + n * kRotMfmaThreads;
    const int i = idx / kD, col = idx % kD;
    float rest = pv[n];
    uint16_t* base = reinterpret_cast<uint16_t*>(&s_B[0][i / 32][col / 16][((i % 32) / 8) * 16 + col % 16]) + (i % 8);
#pragma unroll
    for (int t = 0; t < kRotTerms; ++t) {
      const uint16_t hb = BF16::round(rest);
      rest -= __uint_as_float((uint32_t)hb << 16);  // exact in fp32
      base[(size_t)t * (sizeof(s_B[0]) / 2)] = hb;
    }
  }
  __syncthreads();

  const int item0 = blockIdx.x * items_per_block;
  const int item1 = min(n_items, item0 + items_per_block);

  // Loads never branch: rows past the block's end re-read its last row (item1 > item0 always)
  // and are simply not stored.  Straight-line loads and stores let the compiler count
  // outstanding memory operations exactly, which keeps the prefetch of the next trip in flight
  // during the matrix work instead of being waited for together with the stores.
  // item -> (batch, row): one scalar division per tile base, then a short carry per lane
  auto split_item = [&](int base, int off, int& b, int& r) {
    b = base / n_new;
    r = base % n_new + off;  // off < 64
    while (r >= n_new) {
      r -= n_new;
      ++b;
    }
  };
  auto load_tile = [&](int t0, uint4 (&raw)[4]) {
    const int itb = min(t0, item1 - 1);
    int b, r;
    split_item(itb, min(t0 + r16, item1 - 1) - itb, b, r);
    const char* src = reinterpret_cast<const char*>(k_new) +
                      ((size_t)(b * Hkv + h) * n_new + r) * (kD * 2) + (size_t)kgrp * 16;
#pragma unroll
    for (int step = 0; step < 4; ++step) raw[step] = load16(src + step * 64);
  };

  constexpr int TPW = kRotMfmaTPW;
  constexpr int kStride = 16 * TPW * kRotMfmaWaves;  // rows the block covers per trip

  // One trip: TPW tiles starting at row t0; FULL = every row of them exists.
  // Results go through the wave's staging tile so that every store instruction writes whole
  // rows (16 bytes per lane, four rows per instruction); stored straight from the accumulator
  // layout a row leaves in 32-byte pieces spread over the trip, which measured 10 % slower.
  // A row of the tile is 256 bytes = 8 units of 32 bytes; unit c of row r sits at unit
  // c ^ ((r >> 1) & 7), which spreads the 8-byte writes (16 rows x one 32-byte unit) and the
  // 16-byte reads over the banks without padding.
  typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
  unsigned char* stage = reinterpret_cast<unsigned char*>(&s_stage[wave][0]);
  auto trip = [&](int t0, const uint4 (&raw)[TPW][4], auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    // The operands in LDS never change, but they must be re-read for every trip: hoisted out of
    // the loop, all 96 of them would live in registers and spill.  An offset the compiler
    // cannot see through (always 0) keeps the reads inside the trip.
    uint32_t opaque = 0;
    __asm__ volatile("" : "+v"(opaque));
    const uint4* bop = &s_B[0][0][0][0] + opaque;
    // P_h is the A operand and the key tile the B operand (the operand layouts are alike, so
    // the LDS image and the key loads are what they would be the other way round): the
    // accumulator of column block nb then holds, for this lane's ONE row r16, the four
    // neighbouring columns 16 nb + 4 kgrp .. + 3, which are packed in registers and leave as one
    // 8-byte LDS store (with the keys as A operand a lane held one column of four rows, and
    // pairing neighbouring columns took a lane exchange and two selects per value).
#pragma unroll
    for (int nb = 0; nb < 8; nb += 2) {
      rot_f32x4_t acc[TPW][2];
#pragma unroll
      for (int u = 0; u < TPW; ++u)
#pragma unroll
        for (int half = 0; half < 2; ++half) acc[u][half] = rot_f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = kRotTerms - 1; t >= 0; --t)  // smallest terms first
#pragma unroll
        for (int step = 0; step < 4; ++step) {
          const rot_bf16x8_t b0 =
              __builtin_bit_cast(rot_bf16x8_t, bop[((t * 4 + step) * 8 + nb) * 64 + lane]);
          const rot_bf16x8_t b1 =
              __builtin_bit_cast(rot_bf16x8_t, bop[((t * 4 + step) * 8 + nb + 1) * 64 + lane]);
#pragma unroll
          for (int u = 0; u < TPW; ++u) {
            const rot_bf16x8_t a = __builtin_bit_cast(rot_bf16x8_t, raw[u][step]);
            acc[u][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b0, a, acc[u][0], 0, 0, 0);
            acc[u][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b1, a, acc[u][1], 0, 0, 0);
          }
        }
#pragma unroll
      for (int u = 0; u < TPW; ++u)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int rt = r16;  // row of the tile
          const int unit = (nb + half) ^ ((rt >> 1) & 7);
          *reinterpret_cast<uint2*>(stage + (u * 16 + rt) * 256 + unit * 32 + kgrp * 8) =
              make_uint2(BF16::round2(acc[u][half][0], acc[u][half][1]),
                         BF16::round2(acc[u][half][2], acc[u][half][3]));
        }
    }
    __builtin_amdgcn_wave_barrier();
    // whole rows out: lane l takes chunk l%16 (8 columns) of row l/16 + 4*pass
    const int itb = min(t0, item1 - 1);
#pragma unroll
    for (int u = 0; u < TPW; ++u)
#pragma unroll
      for (int pass = 0; pass < 4; ++pass) {
        const int rt = 4 * pass + kgrp, c = r16;
        const int it = t0 + 16 * u + rt;
        int b, r;
        split_item(itb, min(it, item1 - 1) - itb, b, r);
        size_t row;
        if constexpr (PAGED) row = (size_t)cache_row(pg, b, h, Hkv, S_cap, pos + r);
        else row = (size_t)(b * Hkv + h) * S_cap + pos + r;
        const int unit = (c >> 1) ^ ((rt >> 1) & 7);
        const u32x4_t val = *reinterpret_cast<const u32x4_t*>(stage + (u * 16 + rt) * 256 + unit * 32 + (c & 1) * 16);
        const int col = 8 * c;
        uint16_t* dst = (col < d) ? klo + row * d + col : khi + row * (kD - d) + (col - d);
        if (FULL || it < item1) *reinterpret_cast<u32x4_t*>(dst) = val;
      }
    __builtin_amdgcn_wave_barrier();
  };

  uint4 nxt[TPW][4];
#pragma unroll
  for (int u = 0; u < TPW; ++u) load_tile(item0 + 16 * (TPW * wave + u), nxt[u]);
  int t0 = item0 + 16 * TPW * wave;
  for (; t0 + 16 * TPW <= item1; t0 += kStride) {  // trips whose rows all exist
    uint4 raw[TPW][4];
#pragma unroll
    for (int u = 0; u < TPW; ++u)
#pragma unroll
      for (int step = 0; step < 4; ++step) raw[u][step] = nxt[u][step];
#pragma unroll
    for (int u = 0; u < TPW; ++u) load_tile(t0 + kStride + 16 * u, nxt[u]);
    trip(t0, raw, std::true_type{});
  }
  if (t0 < item1) trip(t0, nxt, std::false_type{});  // ragged last trip of this wave
}

hipError_t launch_rotate(const Shape& s, const void* k_new, const float* P, void* klo, void* khi,
                         int pos, int n_new, hipStream_t st) {
  const bool paged = s.pg.table != nullptr;
  const long long n_items_ll = (long long)s.B * n_new;
  if (n_items_ll > 0x7fffffffLL) return hipErrorInvalidValue;
  const int n_items = (int)n_items_ll;
  if (s.dtype == 1) {
    // One block per CU where the rows allow it: a block's set-up (P_h split into LDS) and its
    // tail are paid once per block, and on the benchmark prefill 8192 rows per block (one round
    // of blocks) took 289 us against 348 us with 2048 (four rounds).
    constexpr int kTripRows = 16 * kRotMfmaTPW * kRotMfmaWaves;
    const int cus = device_cus();
    long long want = (n_items_ll * s.Hkv + cus - 1) / cus;
    want = (want + kTripRows - 1) / kTripRows * kTripRows;
    int ipb_m = (int)(want < kRotMfmaMinItems ? kRotMfmaMinItems : want > kRotMfmaMaxItems ? kRotMfmaMaxItems : want);
    if (n_items < ipb_m) ipb_m = ((n_items + 15) / 16) * 16;
    dim3 grid_m((n_items + ipb_m - 1) / ipb_m, s.Hkv);
    if (paged)
      hipLaunchKernelGGL(rotate_mfma_kernel<true>, grid_m, dim3(kRotMfmaThreads), 0, st,
                         static_cast<const uint16_t*>(k_new), P, static_cast<uint16_t*>(klo),
                         static_cast<uint16_t*>(khi), s.Hkv, s.S_cap, s.d, pos, n_new, n_items, ipb_m,
                         s.pg);
    else
      hipLaunchKernelGGL(rotate_mfma_kernel<false>, grid_m, dim3(kRotMfmaThreads), 0, st,
                         static_cast<const uint16_t*>(k_new), P, static_cast<uint16_t*>(klo),
                         static_cast<uint16_t*>(khi), s.Hkv, s.S_cap, s.d, pos, n_new, n_items, ipb_m,
                         s.pg);
    return hipGetLastError();
  }
  // fp32 caches: the vector kernel (P_h in LDS as fp32)
  int ipb = 512;
  if (n_items < ipb) ipb = ((n_items + kRotTile - 1) / kRotTile) * kRotTile;
  const dim3 grid((n_items + ipb - 1) / ipb, s.Hkv);
  hipLaunchKernelGGL(rotate_kernel<F32>, grid, dim3(kRotThreads), 0, st,
                     static_cast<const float*>(k_new), P, static_cast<float*>(klo),
                     static_cast<float*>(khi), s.Hkv, s.S_cap, s.d, pos, n_new, n_items, ipb, s.pg);
  return hipGetLastError();
}

}  // namespace loki
