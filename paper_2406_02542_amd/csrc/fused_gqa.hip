// The whole decode step of Loki (Algorithm 1 lines 3 and 5-9 of arXiv 2406.02542) for one
// (batch, KV head) unit whose G > 1 query heads share ONE selection (one index set per KV head,
// ranked by the maximum of the group's approximate scores), in ONE block, bf16 cache:
//   rotate the G queries; score the low-rank slab on the matrix cores (score_mfma_impl.h) and
//   keep the group maximum of every row in LDS; select the top-k in LDS (select_impl.h); attend
//   over the selected rows for all G heads on the matrix cores (attend_mfma_impl.h).
// No score, index list or partial result leaves the CU and there is no launch boundary, so the
// select stage of one block overlaps the memory stages of the block it shares the CU with.
// The stages use LDS one after the other: the rotation's partial sums, then the scores, then
// the value tiles of the attention stage and finally the merge of the waves share one region.
#include "fused_gqa_impl.h"

namespace loki {

#ifdef LOKI_PHASE_TIMING
extern "C" int loki_debug_read_gqa_ts(unsigned long long* host_dst, size_t count) {
  return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(loki::g_phase_ts), count * sizeof(unsigned long long));
}
#endif

// ---- host side ---------------------------------------------------------------------------------
bool fused_gqa_eligible(const Shape& s, int select_mode) {
  if (s.dtype != 1 || select_mode != 1) return false;
  if (s.G != 2 && s.G != 4 && s.G != 8) return false;
  if (s.rg.queries > 1) return false;
  if (s.pg.table != nullptr && s.pg.pages_per_seq > kGqaMaxPages) return false;  // page list in LDS
  const int nch = s.d / 8;
  if (s.d % 8 != 0 || (nch & (nch - 1)) != 0 || nch < 2 || s.d >= kD) return false;
  return s.S <= 16384 && s.k <= kGqaMaxK;
}

bool fused_gqa_preferred(const Shape& s, int select_mode) {
  if (!fused_gqa_eligible(s, select_mode)) return false;
  // one block per unit: worth it from a quarter of the CUs on (three eighths for sequences
  // beyond 8192 rows); below that the split path's many blocks per unit win (measured at 16 to
  // 192 units, S = 4096 / 8192 / 16384, 4 and 8 query heads per KV head)
  const long long units = (long long)s.B * s.Hkv, cus = device_cus();
  return s.S <= 8192 ? 4 * units >= cus : 8 * units >= 3 * cus;
}

template <int THREADS, int NCH, int G, int KPT, bool PAGED = false>
static hipError_t launch_fused_gqa_k(const Shape& s, const void* q, const float* P, const void* klo,
                                     const void* khi, const void* v, void* out, int32_t* out_idx,
                                     hipStream_t st) {
  auto kern = fused_gqa_kernel<THREADS, NCH, G, KPT, PAGED>;
  const size_t lds = GqaLds<THREADS, G>::total_bytes(s.S, s.k);
  static std::atomic<unsigned long long> lds_allowed{0};  // per instantiation: devices already set up
  const hipError_t e = allow_dynamic_lds(
      reinterpret_cast<const void*>(kern),
      (int)GqaLds<THREADS, G>::total_bytes(THREADS == 256 ? 8192 : 16384, kGqaMaxK), lds_allowed);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(s.B * s.Hkv), dim3(THREADS), lds, st,
                     static_cast<const uint16_t*>(klo), static_cast<const uint16_t*>(khi),
                     static_cast<const uint16_t*>(v), static_cast<const uint16_t*>(q), P,
                     static_cast<uint16_t*>(out), out_idx, s.Hkv, s.S, s.S_cap, s.k, s.rg, s.ap, s.pg,
                     ClusterArgs{});
  return hipGetLastError();
}

template <int NCH, int G>
static hipError_t launch_fused_gqa_g(const Shape& s, const void* q, const float* P, const void* klo,
                                     const void* khi, const void* v, void* out, int32_t* out_idx,
                                     hipStream_t st) {
  // 256 threads when two blocks have to share a CU; 512 when a block has a CU to itself anyway
  // (a unit's time is set by the instructions its waves issue, so twice the waves per unit are
  // faster: 8 query heads, S = 8192, 128 units: 45 -> 39 us)
  const bool alone = s.B * s.Hkv <= device_cus();
  if (s.pg.table != nullptr) {  // (a paged cache: two block shapes)
    if (s.S > 256 * 32 || alone)
      return launch_fused_gqa_k<512, NCH, G, 32, true>(s, q, P, klo, khi, v, out, out_idx, st);
    return launch_fused_gqa_k<256, NCH, G, 32, true>(s, q, P, klo, khi, v, out, out_idx, st);
  }
  if (s.S > 256 * 32 || alone) return launch_fused_gqa_k<512, NCH, G, 32>(s, q, P, klo, khi, v, out, out_idx, st);
  if (s.S <= 256 * 16) return launch_fused_gqa_k<256, NCH, G, 16>(s, q, P, klo, khi, v, out, out_idx, st);
  return launch_fused_gqa_k<256, NCH, G, 32>(s, q, P, klo, khi, v, out, out_idx, st);
}

template <int NCH>
static hipError_t launch_fused_gqa_n(const Shape& s, const void* q, const float* P, const void* klo,
                                     const void* khi, const void* v, void* out, int32_t* out_idx,
                                     hipStream_t st) {
  switch (s.G) {
    case 2: return launch_fused_gqa_g<NCH, 2>(s, q, P, klo, khi, v, out, out_idx, st);
    case 4: return launch_fused_gqa_g<NCH, 4>(s, q, P, klo, khi, v, out, out_idx, st);
    case 8: return launch_fused_gqa_g<NCH, 8>(s, q, P, klo, khi, v, out, out_idx, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_fused_gqa(const Shape& s, const void* q, const float* P, const void* klo,
                            const void* khi, const void* v, void* out, int32_t* out_idx,
                            hipStream_t st) {
  if (!fused_gqa_eligible(s, 1)) return hipErrorInvalidValue;
  switch (s.d / 8) {
    case 2: return launch_fused_gqa_n<2>(s, q, P, klo, khi, v, out, out_idx, st);
    case 4: return launch_fused_gqa_n<4>(s, q, P, klo, khi, v, out, out_idx, st);
    case 8: return launch_fused_gqa_n<8>(s, q, P, klo, khi, v, out, out_idx, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace loki
