// The single-launch grouped-query decode step (fused_gqa_impl.h) for launches with fewer
// (batch, KV head) units than the chip has compute units: C = 2, 4 or 8 blocks share a unit,
// each on a slice of its rows, so that the launch covers the chip.  The blocks of a unit find
// the top-k threshold together (cluster_impl.h: Algorithm 1 line 6 of arXiv 2406.02542 over
// rows that live in different blocks) and the last one to finish merges the attention partials
// (lines 7-9).
#include "fused_gqa_impl.h"

namespace loki {

constexpr int kClusterThreads = 512;
constexpr int kClusterKpt = 32;
constexpr int kClusterMaxSlice = kClusterThreads * kClusterKpt;  // rows whose keys fit the block's LDS
constexpr int kClusterMaxList = 8192;                            // selected rows one block may end up with

#ifdef LOKI_PHASE_TIMING
extern "C" int loki_debug_read_cluster_ts(unsigned long long* host_dst, size_t count) {
  return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(loki::g_phase_ts), count * sizeof(unsigned long long));
}
#endif

// Clears the control words that must start at zero: every block's arrival flag and the ticket
// of every unit (one word in each kClusterFlagStride words), and the error word behind the
// last unit a launch can have.
__global__ void cluster_reset_kernel(uint32_t* counters, int units) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int n = units * (kClusterMax + 1);
  if (i < n) counters[(size_t)i * kClusterFlagStride] = 0u;
  if (i == n) counters[(size_t)kClusterMaxUnits * kClusterCounterStride] = 0u;
}

static inline int cluster_padded_units(const Shape& s) { return (s.B * s.Hkv + 7) / 8 * 8; }

int fused_gqa_cluster_blocks(const Shape& s, int select_mode) {
  if (s.dtype != 1 || select_mode != 1) return 0;
  if (s.G != 2 && s.G != 4 && s.G != 8) return 0;
  const int nch = s.d / 8;
  if (s.d % 8 != 0 || (nch & (nch - 1)) != 0 || nch < 2 || s.d >= kD) return 0;
  // every block of the launch must be resident at once (the blocks of a unit wait for each
  // other): one block per compute unit at most
  const int padded = cluster_padded_units(s), cus = device_cus();
  if (s.B * s.Hkv > kClusterMaxUnits) return 0;
  int C = 1;
  while (2 * C <= kClusterMax && padded * 2 * C <= cus) C *= 2;
  if (C < 2) return 0;
  const int L = gqa_slice_rows(s.S, C);
  if (L > kClusterMaxSlice || (s.k < L ? s.k : L) > kClusterMaxList) return 0;
  return C;
}

bool fused_gqa_cluster_eligible(const Shape& s, int select_mode) {
  if (s.rg.queries > 1) return false;
  if (s.pg.table != nullptr && s.pg.pages_per_seq > kGqaMaxPages) return false;  // page list in LDS
  return fused_gqa_cluster_blocks(s, select_mode) > 0;
}

bool fused_gqa_cluster_preferred(const Shape& s, int select_mode) {
  if (!fused_gqa_cluster_eligible(s, select_mode)) return false;
  // The exchanges between a unit's blocks cost about 10 us; they pay off once a unit has enough
  // rows or moves enough bytes (measured at 16 to 128 units, 2, 4 and 8 query heads per KV head:
  // from S = 12288 on the cluster is level with or up to 25 % faster than the better of the other
  // two sequences; at S = 8192, k = 1024, d = 32, 1 MB a unit, it is 3 to 10 % slower).
  const long long unit_bytes = (long long)s.S * s.d * 2 + (long long)s.k * kD * 4;
  return s.S >= 12288 || unit_bytes >= 1310720;
}

static std::atomic<uint32_t> g_spin_limit{kClusterSpinLimit};
void set_cluster_spin_limit(uint32_t polls) { g_spin_limit.store(polls, std::memory_order_relaxed); }

namespace {
struct ClusterPlan {
  size_t xhist, xcand, partial, total;  // byte offsets
};
ClusterPlan cluster_plan(const Shape& s, int C) {
  const size_t units = (size_t)s.B * s.Hkv;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  ClusterPlan p;
  size_t off = 0;
  p.xhist = off;
  off += up(units * kClusterRounds * C * kClusterThreads * kClusterSlotBytes);
  p.xcand = off;
  off += up(units * (size_t)GqaLds<kClusterThreads, 2, true>::kCandCap * 4);
  p.partial = off;
  off += up(units * s.G * C * (size_t)kPartialStride * 4);
  p.total = off;
  return p;
}
}  // namespace

size_t fused_gqa_cluster_bytes(const Shape& s, int select_mode) {
  const int C = fused_gqa_cluster_blocks(s, select_mode);
  return C ? cluster_plan(s, C).total : 0;
}

template <int NCH, int G, bool PAGED>
static hipError_t launch_cluster_k(const Shape& s, int C, const void* q, const float* P, const void* klo,
                                   const void* khi, const void* v, void* out, int32_t* out_idx,
                                   uint32_t* ctl, bool ctl_clean, void* region, uint32_t spin_limit,
                                   hipStream_t st) {
  using Lds = GqaLds<kClusterThreads, G, true>;
  auto kern = fused_gqa_kernel<kClusterThreads, NCH, G, kClusterKpt, PAGED, true>;
  const int L = gqa_slice_rows(s.S, C);
  const size_t lds = Lds::total_bytes(L, s.k < L ? s.k : L);
  static std::atomic<unsigned long long> lds_allowed{0};  // per instantiation: devices already set up
  const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern),
                                         (int)Lds::total_bytes(kClusterMaxSlice, kClusterMaxList), lds_allowed);
  if (e != hipSuccess) return e;
  const ClusterPlan p = cluster_plan(s, C);
  char* base = static_cast<char*>(region);
  ClusterArgs cl;
  cl.counters = ctl;
  cl.error = ctl + (size_t)kClusterMaxUnits * kClusterCounterStride;
  cl.xhist = reinterpret_cast<uint32_t*>(base + p.xhist);
  cl.xhist_bytes = p.xcand - p.xhist;
  cl.xcand = reinterpret_cast<uint32_t*>(base + p.xcand);
  cl.xcand_bytes = p.partial - p.xcand;
  cl.partial = reinterpret_cast<float*>(base + p.partial);
  cl.C = C;
  cl.units = s.B * s.Hkv;
  cl.spin_limit = spin_limit;
  // the arrival flags and tickets start at zero: unless the caller vouches for the workspace,
  // clear them (with a kernel, not a memset: a caller may be capturing the stream into a graph)
  if (!ctl_clean) {
    const int n_zero = cl.units * (kClusterMax + 1) + 1;
    hipLaunchKernelGGL(cluster_reset_kernel, dim3((n_zero + 255) / 256), dim3(256), 0, st, cl.counters, cl.units);
  }
  hipLaunchKernelGGL(kern, dim3(cluster_padded_units(s) * C), dim3(kClusterThreads), lds, st,
                     static_cast<const uint16_t*>(klo), static_cast<const uint16_t*>(khi),
                     static_cast<const uint16_t*>(v), static_cast<const uint16_t*>(q), P,
                     static_cast<uint16_t*>(out), out_idx, s.Hkv, s.S, s.S_cap, s.k, s.rg, s.ap, s.pg, cl);
  return hipGetLastError();
}

template <int NCH>
static hipError_t launch_cluster_n(const Shape& s, int C, const void* q, const float* P, const void* klo,
                                   const void* khi, const void* v, void* out, int32_t* out_idx,
                                   uint32_t* ctl, bool ctl_clean, void* region, uint32_t spin_limit,
                                   hipStream_t st) {
#define LOKI_CLUSTER_G(Gn)                                                                              \
  case Gn:                                                                                              \
    return s.pg.table != nullptr                                                                        \
               ? launch_cluster_k<NCH, Gn, true>(s, C, q, P, klo, khi, v, out, out_idx, ctl, ctl_clean, region, \
                                                 spin_limit, st)                                        \
               : launch_cluster_k<NCH, Gn, false>(s, C, q, P, klo, khi, v, out, out_idx, ctl, ctl_clean, region, \
                                                  spin_limit, st)
  switch (s.G) {
    LOKI_CLUSTER_G(2);
    LOKI_CLUSTER_G(4);
    LOKI_CLUSTER_G(8);
    default: return hipErrorInvalidValue;
  }
#undef LOKI_CLUSTER_G
}

hipError_t launch_fused_gqa_cluster(const Shape& s, const void* q, const float* P, const void* klo,
                                    const void* khi, const void* v, void* out, int32_t* out_idx,
                                    uint32_t* ctl, bool ctl_clean, void* region, hipStream_t st) {
  if (!fused_gqa_cluster_eligible(s, 1) || region == nullptr || ctl == nullptr) return hipErrorInvalidValue;
  const int C = fused_gqa_cluster_blocks(s, 1);
  const uint32_t spin_limit = g_spin_limit.load(std::memory_order_relaxed);
  switch (s.d / 8) {
    case 2: return launch_cluster_n<2>(s, C, q, P, klo, khi, v, out, out_idx, ctl, ctl_clean, region, spin_limit, st);
    case 4: return launch_cluster_n<4>(s, C, q, P, klo, khi, v, out, out_idx, ctl, ctl_clean, region, spin_limit, st);
    case 8: return launch_cluster_n<8>(s, C, q, P, klo, khi, v, out, out_idx, ctl, ctl_clean, region, spin_limit, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace loki
