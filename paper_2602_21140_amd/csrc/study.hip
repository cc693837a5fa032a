// Activation counting for the lost-expert study (paper Sec. 4.2: experts are ranked by how
// often they are activated, per layer and aggregated, to choose which ones to fail).
#include <algorithm>

#include "ctx.hpp"

namespace revive {

namespace {

// Per-workgroup LDS histogram of the selected expert ids, then one 64-bit atomic add per expert
// and workgroup.  Integer addition: the result does not depend on the order of the adds.
__global__ __launch_bounds__(256) void expert_counts_kernel(const int32_t* __restrict__ topk_logical, int n, int E,
                                                            unsigned long long* __restrict__ counts) {
  __shared__ int hist[kMaxE];
  for (int e = threadIdx.x; e < E; e += 256) hist[e] = 0;
  __syncthreads();
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) {
    const int e = topk_logical[i];
    if (e >= 0 && e < E) atomicAdd(&hist[e], 1);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += 256)
    if (hist[e]) atomicAdd(&counts[e], static_cast<unsigned long long>(hist[e]));
}

}  // namespace

int launch_expert_counts(revive_ctx* ctx, const int32_t* topk_logical, int T, int64_t* counts, hipStream_t stream) {
  const int n = T * ctx->cfg.k;
  const int grid = std::min(1024, ceil_div(n, 256 * 4));
  KernelTimer timer(ctx, REVIVE_K_EXPERT_COUNTS, stream);
  hipLaunchKernelGGL(expert_counts_kernel, dim3(std::max(1, grid)), dim3(256), 0, stream, topk_logical, n, ctx->cfg.E,
                     reinterpret_cast<unsigned long long*>(counts));
  return check_hip(ctx, hipGetLastError(), "expert_counts launch");
}

}  // namespace revive
