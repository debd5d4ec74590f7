// Per-head top-k selection (Algorithm 1 line 6 of arXiv 2406.02542) as a stand-alone kernel:
// one 1024-thread block per selecting head reads that head's approximate scores and writes
// the k selected positions (ascending) together with their scores, which the attention
// stage reuses as the low-rank part of the exact logits.
#include "select_impl.h"

namespace loki {

constexpr int kSelThreads = 1024;

__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ scores,
                                                             int32_t* __restrict__ sel_idx,
                                                             float* __restrict__ sel_score, int S,
                                                             int k) {
  __shared__ SelectSmem<kSelThreads> sm;
  const float* a = scores + (size_t)blockIdx.x * S;
  int32_t* out = sel_idx + (size_t)blockIdx.x * k;
  float* outs = sel_score + (size_t)blockIdx.x * k;
  block_select_topk<kSelThreads>(a, S, k, sm, [&](int rank, int pos) {
    out[rank] = pos;
    outs[rank] = a[pos];
  });
}

hipError_t launch_select(const Shape& s, int n_sel_heads, const float* scores, int32_t* sel_idx,
                         float* sel_score, hipStream_t st) {
  hipLaunchKernelGGL(select_kernel, dim3(n_sel_heads), dim3(kSelThreads), 0, st, scores, sel_idx,
                     sel_score, s.S, s.k);
  return hipGetLastError();
}

}  // namespace loki
