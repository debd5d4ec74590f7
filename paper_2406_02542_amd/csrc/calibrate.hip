// Calibration and diagnostics around the decode path (arXiv 2406.02542, Section 3.1): the PCA
// of a set of calibration keys that produces the per-head basis P, Rank@v of its spectrum
// (Eq. 2), and the Jaccard agreement of two index lists (the quantity of Figure 6, left).
//
//   gram_kernel        (chunk, head)  G = sum_s k_s^T k_s and column sums over a run of rows, on
//                                     the matrix cores: a 32-row tile is written transposed into
//                                     LDS (swizzled, see gram_swizzle) so that both operands of
//                                     v_mfma_f32_16x16x32_bf16 (eight consecutive rows of one
//                                     column per lane) are one 16-byte LDS read; bf16 keys are exact, fp32 keys enter as two bf16 terms
//   cov_reduce_kernel  (head)         chunk partials added in a fixed order in fp64; sample
//                                     covariance C = (G - s s^T / N) / (N - 1)
//   jacobi_sweep_kernel, jacobi_apply_kernel, jacobi_finish_kernel
//                                     cyclic Jacobi eigensolver in fp64 (see there): C resident in
//                                     LDS (129 KiB), 64 disjoint rotations per round in a
//                                     round-robin order, the eigenvector accumulation spread over
//                                     8 blocks per head; eigenpairs sorted by decreasing
//                                     eigenvalue, every component's largest entry made positive
//   rank_at_kernel, layer_width_kernel, jaccard_kernel    small reductions
#include "common.h"

namespace loki {

typedef __bf16 cal_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float cal_f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kGramThreads = 256;
constexpr int kGramTile = 32;    // rows per tile = the k dimension of one MFMA
constexpr int kGramPitch = 144;  // bytes per column of the transposed tile: 8 slots of 16 bytes + 16
// A column's four 16-byte granules (rows 8 g .. 8 g + 7) sit in slots g ^ gram_swizzle(column).
// Columns one 16-byte chunk of a key row apart (8 columns) are written by neighbouring lanes in
// the same instruction and lie a multiple of 128 bytes apart whatever the pitch, i.e. in the same
// bank; the swizzle spreads the 16 chunks of a row over 8 bank groups (2-way instead of 16-way
// conflicts of the 2-byte transposing writes).
__device__ __forceinline__ int gram_swizzle(int col) { return (col >> 3) & 7; }

// NT = bf16 terms per element: 1 for bf16 storage, 2 for fp32 storage (value, remainder).
template <int NT>
__global__ __launch_bounds__(kGramThreads) void gram_kernel(const void* __restrict__ keys,
                                                            float* __restrict__ gram_part,
                                                            float* __restrict__ sum_part,
                                                            long long N, int rows_per_chunk) {
  constexpr int kColsPerChunk = NT == 1 ? 8 : 4;          // columns in a 16-byte chunk
  constexpr int kChunksPerRow = kD / kColsPerChunk;       // 16 or 32
  constexpr int kRowsPerPass = kGramThreads / kChunksPerRow;  // 16 or 8
  constexpr int kPasses = kGramTile / kRowsPerPass;       // 2 or 4
  __shared__ __align__(16) unsigned char s_t[NT][kD * kGramPitch];
  __shared__ float s_sum[kRowsPerPass][kD];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kgrp = lane >> 4;
  const int chunk = blockIdx.x, head = blockIdx.y, nchunks = gridDim.x;
  const long long r0 = (long long)chunk * rows_per_chunk;
  const long long r1 = min(N, r0 + rows_per_chunk);
  const int c = tid % kChunksPerRow, rr = tid / kChunksPerRow;
  const size_t row_bytes = (size_t)kD * (NT == 1 ? 2 : 4);
  const char* base = static_cast<const char*>(keys) + (size_t)head * N * row_bytes + (size_t)c * 16;

  cal_f32x4_t acc[2][8];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = cal_f32x4_t{0.f, 0.f, 0.f, 0.f};
  float csum[kColsPerChunk];
#pragma unroll
  for (int e = 0; e < kColsPerChunk; ++e) csum[e] = 0.f;

  auto load_tile = [&](long long t0, uint4 (&raw)[kPasses]) {
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const long long row = t0 + p * kRowsPerPass + rr;
      raw[p] = row < r1 ? load16(base + (size_t)row * row_bytes) : make_uint4(0, 0, 0, 0);
    }
  };

  uint4 raw[kPasses];
  load_tile(r0, raw);
  for (long long t0 = r0; t0 < r1; t0 += kGramTile) {
    __syncthreads();  // the previous tile's operand reads are done
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int row = p * kRowsPerPass + rr;  // row inside the tile
      if constexpr (NT == 1) {
        float f[8];
        BF16::unpack(raw[p], f);
        const uint32_t w[4] = {raw[p].x, raw[p].y, raw[p].z, raw[p].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          csum[e] += f[e];
          const uint16_t h = (uint16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu));
          *reinterpret_cast<uint16_t*>(&s_t[0][(8 * c + e) * kGramPitch + (((row >> 3) ^ gram_swizzle(8 * c + e)) << 4) + (row & 7) * 2]) = h;
        }
      } else {
        float f[4];
        F32::unpack(raw[p], f);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          csum[e] += f[e];
          const uint16_t hi = BF16::round(f[e]);
          const uint16_t lo = BF16::round(f[e] - __uint_as_float((uint32_t)hi << 16));
          *reinterpret_cast<uint16_t*>(&s_t[0][(4 * c + e) * kGramPitch + (((row >> 3) ^ gram_swizzle(4 * c + e)) << 4) + (row & 7) * 2]) = hi;
          *reinterpret_cast<uint16_t*>(&s_t[NT - 1][(4 * c + e) * kGramPitch + (((row >> 3) ^ gram_swizzle(4 * c + e)) << 4) + (row & 7) * 2]) = lo;
        }
      }
    }
    __syncthreads();
    load_tile(t0 + kGramTile, raw);  // next tile's loads fly during the products (zeros past the end)
    // wave w owns output rows 32 w .. 32 w + 31 (two 16-row tiles) of all 128 columns
    cal_bf16x8_t a[NT][2];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int i = 0; i < 2; ++i)
        a[t][i] = *reinterpret_cast<const cal_bf16x8_t*>(
            &s_t[t][(32 * wave + 16 * i + r16) * kGramPitch + ((kgrp ^ gram_swizzle(32 * wave + 16 * i + r16)) << 4)]);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      cal_bf16x8_t b[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t)
        b[t] = *reinterpret_cast<const cal_bf16x8_t*>(
            &s_t[t][(16 * j + r16) * kGramPitch + ((kgrp ^ gram_swizzle(16 * j + r16)) << 4)]);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        if constexpr (NT == 2) {  // smallest terms first; remainder x remainder is below fp32's last place
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[1][i], b[0], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[0][i], b[1], acc[i][j], 0, 0, 0);
        }
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[0][i], b[0], acc[i][j], 0, 0, 0);
      }
    }
  }

  // partial Gram matrix: lane holds rows 4 kgrp + e, column r16 of each 16 x 16 tile
  float* gp = gram_part + ((size_t)head * nchunks + chunk) * kD * kD;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        gp[(size_t)(32 * wave + 16 * i + 4 * kgrp + e) * kD + 16 * j + r16] = acc[i][j][e];
  // column sums: the kRowsPerPass threads that share a chunk are added in a fixed order
#pragma unroll
  for (int e = 0; e < kColsPerChunk; ++e) s_sum[rr][kColsPerChunk * c + e] = csum[e];
  __syncthreads();
  if (tid < kD) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < kRowsPerPass; ++r) s += s_sum[r][tid];
    sum_part[((size_t)head * nchunks + chunk) * kD + tid] = s;
  }
}

// C = (G - s s^T / N) / (N - 1), chunk partials added in order in fp64.
__global__ __launch_bounds__(1024) void cov_reduce_kernel(const float* __restrict__ gram_part,
                                                          const float* __restrict__ sum_part,
                                                          double* __restrict__ cov, long long N,
                                                          int nchunks) {
  const int head = blockIdx.x, e = blockIdx.y * 1024 + threadIdx.x;  // entry (row, col)
  const int row = e / kD, col = e % kD;
  const float* gp = gram_part + (size_t)head * nchunks * kD * kD;
  const float* sp = sum_part + (size_t)head * nchunks * kD;
  double g = 0.0, sr = 0.0, sc = 0.0;
  for (int cc = 0; cc < nchunks; ++cc) {
    g += (double)gp[(size_t)cc * kD * kD + e];
    sr += (double)sp[cc * kD + row];
    sc += (double)sp[cc * kD + col];
  }
  const double n = (double)N;
  cov[(size_t)head * kD * kD + e] = (g - sr * sc / n) / (n > 1.0 ? n - 1.0 : 1.0);
}

// ---- eigensolver ------------------------------------------------------------------------------
// Cyclic Jacobi in fp64, one sweep (127 rounds of 64 disjoint rotations, round-robin pairing)
// per launch pair:
//   jacobi_sweep_kernel (head)            C resident in LDS (129 KiB); checks convergence, then
//                                         rotates C round by round and logs every rotation's
//                                         (cos, sin); C goes back to global memory for the next sweep
//   jacobi_apply_kernel (column slice, head)  the eigenvector accumulator Vt is only ever rotated,
//                                         row pair by row pair, and columns do not mix: each block
//                                         keeps 16 columns of Vt in LDS and replays the sweep's log
// so that the accumulation, which used to cost the solver block 256 KiB of L2 traffic per round,
// is spread over 8 blocks per head.  The host enqueues kJacMaxSweeps pairs; a converged head's
// blocks leave at once.  jacobi_finish_kernel sorts the eigenpairs and writes P.
constexpr int kJacThreads = 1024;
constexpr int kJacPitch = kD + 1;  // doubles per row of the LDS-resident matrix
constexpr int kJacMaxSweeps = 30;
constexpr int kJacRounds = kD - 1;
constexpr int kJacSliceCols = 16;                  // columns of Vt one apply block owns
constexpr int kJacSlices = kD / kJacSliceCols;
constexpr int kJacApplyThreads = 256;

// round-robin pairing of 128 indices: slot 0 pairs (round, 127), slot t pairs
// ((round + t) % 127, (round - t) % 127); returned with p < q
__device__ __forceinline__ void jacobi_pair(int round, int slot, int& p, int& q) {
  if (slot == 0) {
    p = round;
    q = kD - 1;
  } else {
    p = (round + slot) % (kD - 1);
    q = (round - slot + (kD - 1)) % (kD - 1);
  }
  if (p > q) {
    const int t = p;
    p = q;
    q = t;
  }
}

// state[head]: 0 while the head still rotates, 1 once it has converged (set here, read by later
// launches); log[head][round][slot] = (cos, sin) of this sweep; n_logged[head] = rounds logged
// by this launch (0 or kJacRounds).
__global__ __launch_bounds__(kJacThreads) void jacobi_sweep_kernel(double* __restrict__ a_all,
                                                                   double2* __restrict__ log_all,
                                                                   int* __restrict__ state,
                                                                   int* __restrict__ n_logged, int sweep) {
  extern __shared__ __align__(16) unsigned char jac_smem[];
  double* A = reinterpret_cast<double*>(jac_smem);  // [128][kJacPitch]
  __shared__ double s_c[kD / 2], s_s[kD / 2];
  __shared__ int s_p[kD / 2], s_q[kD / 2];
  __shared__ double s_red[kJacThreads / 64];

  const int tid = threadIdx.x, head = blockIdx.x;
  if (sweep == 0 && tid == 0) state[head] = 0;
  if (sweep > 0 && state[head] != 0) {  // (uniform; written by an earlier launch)
    if (tid == 0) n_logged[head] = 0;
    return;
  }
  double* Ag = a_all + (size_t)head * kD * kD;
  double2* log = log_all + (size_t)head * kJacRounds * (kD / 2);
  for (int e = tid; e < kD * kD; e += kJacThreads) A[(e / kD) * kJacPitch + e % kD] = Ag[e];
  __syncthreads();

  auto block_sum = [&](double x) -> double {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    __syncthreads();
    if ((tid & 63) == 0) s_red[tid >> 6] = x;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < kJacThreads / 64; ++w) t += s_red[w];
    return t;
  };

  // converged when the off-diagonal mass is at rounding level of the diagonal's
  double off = 0.0, dg = 0.0;
  for (int e = tid; e < kD * kD; e += kJacThreads) {
    const double x = A[(e / kD) * kJacPitch + e % kD];
    if (e / kD == e % kD) dg += x * x; else off += x * x;
  }
  off = block_sum(off);
  dg = block_sum(dg);
  if (off <= 1e-28 * dg || dg == 0.0) {  // uniform: every thread holds the same sums
    if (tid == 0) {
      state[head] = 1;
      n_logged[head] = 0;
    }
    return;
  }

  for (int round = 0; round < kJacRounds; ++round) {
    if (tid < kD / 2) {
      int p, q;
      jacobi_pair(round, tid, p, q);
      const double app = A[p * kJacPitch + p], aqq = A[q * kJacPitch + q], apq = A[p * kJacPitch + q];
      double cs = 1.0, sn = 0.0;
      if (fabs(apq) > 1e-300) {
        const double theta = (aqq - app) / (2.0 * apq);
        const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
        cs = 1.0 / sqrt(t * t + 1.0);
        sn = t * cs;
      }
      s_p[tid] = p; s_q[tid] = q; s_c[tid] = cs; s_s[tid] = sn;
      log[round * (kD / 2) + tid] = make_double2(cs, sn);
    }
    __syncthreads();
    // A <- J^T A J, one 2 x 2 block (row pair, column pair) at a time: the rows are rotated
    // first and the columns after, element by element the same operations as two whole-matrix
    // passes, with every element read and written once
    for (int it = tid; it < (kD / 2) * (kD / 2); it += kJacThreads) {
      const int pr = it / (kD / 2), pc = it % (kD / 2);
      const int p = s_p[pr], q = s_q[pr], p2 = s_p[pc], q2 = s_q[pc];
      const double cs = s_c[pr], sn = s_s[pr], cs2 = s_c[pc], sn2 = s_s[pc];
      const double xpp = A[p * kJacPitch + p2], xpq = A[p * kJacPitch + q2];
      const double xqp = A[q * kJacPitch + p2], xqq = A[q * kJacPitch + q2];
      const double tpp = cs * xpp - sn * xqp, tqp = sn * xpp + cs * xqp;  // rows p, q at column p2
      const double tpq = cs * xpq - sn * xqq, tqq = sn * xpq + cs * xqq;  // rows p, q at column q2
      A[p * kJacPitch + p2] = cs2 * tpp - sn2 * tpq;
      A[p * kJacPitch + q2] = sn2 * tpp + cs2 * tpq;
      A[q * kJacPitch + p2] = cs2 * tqp - sn2 * tqq;
      A[q * kJacPitch + q2] = sn2 * tqp + cs2 * tqq;
    }
    __syncthreads();
  }
  for (int e = tid; e < kD * kD; e += kJacThreads) Ag[e] = A[(e / kD) * kJacPitch + e % kD];
  if (tid == 0) n_logged[head] = kJacRounds;
}

// Vt[j][i] = component j, entry i.  Block (slice, head) owns entries i in [16 slice, 16 slice + 16)
// of every component; the rotation of components p and q is the same on every entry.  The first
// sweep starts from the identity.
__global__ __launch_bounds__(kJacApplyThreads) void jacobi_apply_kernel(double* __restrict__ vt_all,
                                                                        const double2* __restrict__ log_all,
                                                                        const int* __restrict__ n_logged,
                                                                        int sweep) {
  __shared__ double s_v[kD][kJacSliceCols + 1];
  const int tid = threadIdx.x, slice = blockIdx.x, head = blockIdx.y;
  const int n_rounds = n_logged[head];
  if (n_rounds == 0 && sweep > 0) return;  // (uniform) nothing to replay: Vt stays as it is
  double* Vt = vt_all + (size_t)head * kD * kD;
  const double2* log = log_all + (size_t)head * kJacRounds * (kD / 2);
  const int i0 = slice * kJacSliceCols;
  for (int e = tid; e < kD * kJacSliceCols; e += kJacApplyThreads) {
    const int j = e / kJacSliceCols, c = e % kJacSliceCols;
    s_v[j][c] = sweep == 0 ? (j == i0 + c ? 1.0 : 0.0) : Vt[(size_t)j * kD + i0 + c];
  }
  __syncthreads();
  // thread t: pair slot t / 4, columns 4 (t % 4) .. + 3 of the slice
  const int slot = tid >> 2, c0 = 4 * (tid & 3);
  for (int round = 0; round < n_rounds; ++round) {
    int p, q;
    jacobi_pair(round, slot, p, q);
    const double2 r = log[round * (kD / 2) + slot];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const double vx = s_v[p][c0 + c], vy = s_v[q][c0 + c];
      s_v[p][c0 + c] = r.x * vx - r.y * vy;
      s_v[q][c0 + c] = r.y * vx + r.x * vy;
    }
    __syncthreads();
  }
  for (int e = tid; e < kD * kJacSliceCols; e += kJacApplyThreads) {
    const int j = e / kJacSliceCols, c = e % kJacSliceCols;
    Vt[(size_t)j * kD + i0 + c] = s_v[j][c];
  }
}

// decreasing eigenvalue order (ties: lower index first); largest entry of a component positive
__global__ __launch_bounds__(kD) void jacobi_finish_kernel(const double* __restrict__ a_all,
                                                           const double* __restrict__ vt_all,
                                                           float* __restrict__ P,
                                                           float* __restrict__ eigenvalues) {
  __shared__ double s_diag[kD];
  const int tid = threadIdx.x, head = blockIdx.x;
  const double* Ag = a_all + (size_t)head * kD * kD;
  const double* Vt = vt_all + (size_t)head * kD * kD;
  s_diag[tid] = Ag[(size_t)tid * kD + tid];
  __syncthreads();
  const double mine = s_diag[tid];
  int rank = 0;
  for (int j = 0; j < kD; ++j) {
    const double other = s_diag[j];
    rank += (other > mine || (other == mine && j < tid)) ? 1 : 0;
  }
  eigenvalues[(size_t)head * kD + rank] = (float)mine;
  const double* vrow = Vt + (size_t)tid * kD;
  double best = 0.0;
  for (int i = 0; i < kD; ++i)
    if (fabs(vrow[i]) > fabs(best)) best = vrow[i];
  const double sgn = best < 0.0 ? -1.0 : 1.0;
  float* Pc = P + (size_t)head * kD * kD + rank;  // column = component
  for (int i = 0; i < kD; ++i) Pc[(size_t)i * kD] = (float)(sgn * vrow[i]);
}

// Eq. 2: the smallest d whose leading normalised eigenvalues sum to at least v percent.
__device__ inline int rank_at_of(const float* __restrict__ lam, int Dn, float v_percent) {
  double total = 0.0;
  for (int i = 0; i < Dn; ++i) total += (double)lam[i];
  double run = 0.0;
  for (int i = 0; i < Dn; ++i) {
    run += (double)lam[i];
    if (run / total >= (double)v_percent / 100.0) return i + 1;
  }
  return Dn;
}

__global__ __launch_bounds__(64) void rank_at_kernel(const float* __restrict__ eigenvalues, int Dn,
                                                     float v_percent, int32_t* __restrict__ ranks) {
  if (threadIdx.x != 0) return;
  ranks[blockIdx.x] = rank_at_of(eigenvalues + (size_t)blockIdx.x * Dn, Dn, v_percent);
}

// Rank_l@v of a layer (the head average of Eq. 2, Section 3.1) and the slab width that the
// variable-width policy of Appendix B.2 derives from it: the average taken up to a whole
// number, then to a multiple of the layout's granularity, at most D.  One block; the ranks are
// integers, so their sum is exact whatever the order.
__global__ __launch_bounds__(256) void layer_width_kernel(const float* __restrict__ eigenvalues,
                                                          int n_heads, int Dn, float v_percent,
                                                          int multiple, float* __restrict__ mean_rank,
                                                          int32_t* __restrict__ d_out) {
  __shared__ int s_sum;
  if (threadIdx.x == 0) s_sum = 0;
  __syncthreads();
  int mine = 0;
  for (int h = threadIdx.x; h < n_heads; h += 256)
    mine += rank_at_of(eigenvalues + (size_t)h * Dn, Dn, v_percent);
  if (mine) atomicAdd(&s_sum, mine);
  __syncthreads();
  if (threadIdx.x == 0) {
    const int sum = s_sum;
    if (mean_rank) *mean_rank = (float)((double)sum / (double)n_heads);
    int d = (sum + n_heads - 1) / n_heads;             // ceil of the average
    d = (d + multiple - 1) / multiple * multiple;
    *d_out = d < Dn ? d : Dn;
  }
}

// |A n B| / |A u B| of two ascending index lists of length k each (entries < 0 are padding).
__global__ __launch_bounds__(256) void jaccard_kernel(const int32_t* __restrict__ a,
                                                      const int32_t* __restrict__ b, int k,
                                                      float* __restrict__ out) {
  __shared__ int s_cnt[3];
  const int32_t* la = a + (size_t)blockIdx.x * k;
  const int32_t* lb = b + (size_t)blockIdx.x * k;
  if (threadIdx.x < 3) s_cnt[threadIdx.x] = 0;
  __syncthreads();
  int inter = 0, na = 0, nb = 0;
  for (int i = threadIdx.x; i < k; i += 256) {
    const int x = la[i];
    nb += lb[i] >= 0 ? 1 : 0;
    if (x < 0) continue;
    ++na;
    int lo = 0, hi = k;  // lower bound of x among the non-negative prefix-ordered entries of b
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      const int y = lb[mid];
      if (y >= 0 && y < x) lo = mid + 1; else hi = mid;
    }
    inter += (lo < k && lb[lo] == x) ? 1 : 0;
  }
  atomicAdd(&s_cnt[0], inter);
  atomicAdd(&s_cnt[1], na);
  atomicAdd(&s_cnt[2], nb);
  __syncthreads();
  if (threadIdx.x == 0) {
    const int uni = s_cnt[1] + s_cnt[2] - s_cnt[0];
    out[blockIdx.x] = uni > 0 ? (float)s_cnt[0] / (float)uni : 1.0f;
  }
}

// ---- launchers ----------------------------------------------------------------------------------
int pca_chunks(int Hkv, long long N, int* rows_per_chunk) {
  long long want = (2 * device_cus() + Hkv - 1) / Hkv;  // about two blocks per CU over all heads
  long long rows = (N + want - 1) / want;
  if (rows < 1024) rows = 1024;
  rows = (rows + kGramTile - 1) / kGramTile * kGramTile;
  *rows_per_chunk = (int)rows;
  return (int)((N + rows - 1) / rows);
}

size_t pca_workspace_bytes(int Hkv, long long N) {
  int rpc;
  const int nc = pca_chunks(Hkv, N, &rpc);
  size_t b = 0;
  b += (size_t)Hkv * nc * kD * kD * sizeof(float);  // partial Gram matrices
  b += (size_t)Hkv * nc * kD * sizeof(float);       // partial column sums
  b = (b + 255) / 256 * 256;
  b += (size_t)Hkv * kD * kD * sizeof(double);      // covariance
  b += (size_t)Hkv * kD * kD * sizeof(double);      // eigenvector accumulator
  b += (size_t)Hkv * kJacRounds * (kD / 2) * sizeof(double2);  // one sweep's rotations
  b += (size_t)2 * Hkv * sizeof(int);               // converged flags, rounds logged
  return b;
}

// stage 0: partial Gram matrices; 1: covariance; 2: eigensolver
hipError_t launch_pca_stage(int stage, int Hkv, int dtype, const void* keys, long long N, float* P,
                            float* eigenvalues, void* workspace, hipStream_t st) {
  int rpc;
  const int nc = pca_chunks(Hkv, N, &rpc);
  char* w = static_cast<char*>(workspace);
  float* gram_part = reinterpret_cast<float*>(w);
  float* sum_part = gram_part + (size_t)Hkv * nc * kD * kD;
  size_t off = ((size_t)Hkv * nc * kD * kD + (size_t)Hkv * nc * kD) * sizeof(float);
  off = (off + 255) / 256 * 256;
  double* cov = reinterpret_cast<double*>(w + off);
  double* vt = cov + (size_t)Hkv * kD * kD;
  if (stage == 0) {
    if (dtype == 0)
      hipLaunchKernelGGL(gram_kernel<2>, dim3(nc, Hkv), dim3(kGramThreads), 0, st, keys, gram_part,
                         sum_part, N, rpc);
    else
      hipLaunchKernelGGL(gram_kernel<1>, dim3(nc, Hkv), dim3(kGramThreads), 0, st, keys, gram_part,
                         sum_part, N, rpc);
  } else if (stage == 1) {
    hipLaunchKernelGGL(cov_reduce_kernel, dim3(Hkv, kD * kD / 1024), dim3(1024), 0, st, gram_part,
                       sum_part, cov, N, nc);
  } else {
    double2* log = reinterpret_cast<double2*>(vt + (size_t)Hkv * kD * kD);
    int* state = reinterpret_cast<int*>(log + (size_t)Hkv * kJacRounds * (kD / 2));
    int* n_logged = state + Hkv;
    const size_t lds = (size_t)kD * kJacPitch * sizeof(double);
    static std::atomic<unsigned long long> lds_allowed{0};  // devices already set up
    const hipError_t ea =
        allow_dynamic_lds(reinterpret_cast<const void*>(jacobi_sweep_kernel), (int)lds, lds_allowed);
    if (ea != hipSuccess) return ea;
    // the covariance array is rotated in place, sweep by sweep
    for (int sweep = 0; sweep < kJacMaxSweeps; ++sweep) {
      hipLaunchKernelGGL(jacobi_sweep_kernel, dim3(Hkv), dim3(kJacThreads), lds, st, cov, log, state,
                         n_logged, sweep);
      hipLaunchKernelGGL(jacobi_apply_kernel, dim3(kJacSlices, Hkv), dim3(kJacApplyThreads), 0, st, vt, log,
                         n_logged, sweep);
    }
    hipLaunchKernelGGL(jacobi_finish_kernel, dim3(Hkv), dim3(kD), 0, st, cov, vt, P, eigenvalues);
  }
  return hipGetLastError();
}

hipError_t launch_rank_at(const float* eigenvalues, int n, int Dn, float v_percent, int32_t* ranks,
                          hipStream_t st) {
  hipLaunchKernelGGL(rank_at_kernel, dim3(n), dim3(64), 0, st, eigenvalues, Dn, v_percent, ranks);
  return hipGetLastError();
}

hipError_t launch_layer_width(const float* eigenvalues, int n, int Dn, float v_percent, int multiple,
                              float* mean_rank, int32_t* d_out, hipStream_t st) {
  hipLaunchKernelGGL(layer_width_kernel, dim3(1), dim3(256), 0, st, eigenvalues, n, Dn, v_percent,
                     multiple, mean_rank, d_out);
  return hipGetLastError();
}

hipError_t launch_jaccard(const int32_t* a, const int32_t* b, int n_lists, int k, float* out,
                          hipStream_t st) {
  hipLaunchKernelGGL(jaccard_kernel, dim3(n_lists), dim3(256), 0, st, a, b, k, out);
  return hipGetLastError();
}

}  // namespace loki
