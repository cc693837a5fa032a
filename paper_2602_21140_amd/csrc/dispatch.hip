// Dispatch (A2E) of the failure-remapped MoE layer: a deterministic stable counting sort of the
// routed rows by physical slot, then the row permutation.
//
// Paper: Sec. 2.3 (dispatch routes tokens to their top-k experts).  Slots are laid out rank by
// rank, so the sorted buffer is rank-segmented: segment r is what rank r would receive.  A failed
// rank's slots never appear in topk_phys (Sec. 3.4), so its segment is empty (Sec. 3.5).
//
// Four kernels, all with grids fixed by T:
//   count    per-chunk LDS histogram of the slot ids               -> block_hist[chunk][P]
//   scan     column scan over chunks, then exclusive scan over P   -> block_hist (bases), slot_offsets
//   place    stable rank of every routed row inside its chunk      -> dst_row, src_of
//   permute  one workgroup per token: read the row once, write it to its k destinations
#include "ctx.hpp"

namespace revive {

namespace {

constexpr int kChunk = kDispatchChunk;  // routed rows per workgroup
constexpr int kThreads = 256;
constexpr int kSteps = kChunk / kThreads;

__global__ __launch_bounds__(kThreads) void dispatch_count_kernel(const int32_t* __restrict__ topk_phys, int N, int P,
                                                                  int32_t* __restrict__ block_hist) {
  __shared__ int hist[kMaxP];
  for (int p = threadIdx.x; p < P; p += kThreads) hist[p] = 0;
  __syncthreads();
  const int base = blockIdx.x * kChunk;
#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    const int i = base + s * kThreads + threadIdx.x;
    if (i < N) {
      const int p = topk_phys[i];
      if (p >= 0 && p < P) atomicAdd(&hist[p], 1);
    }
  }
  __syncthreads();
  for (int p = threadIdx.x; p < P; p += kThreads) block_hist[static_cast<int64_t>(blockIdx.x) * P + p] = hist[p];
}

// One workgroup of 1024 threads.  Thread p turns column p of block_hist into exclusive running
// sums over the chunks (the rows of slot p that earlier chunks hold); the totals are then scanned
// over p.  slot_offsets[P] = number of valid routed rows.
__global__ __launch_bounds__(kMaxP) void dispatch_scan_kernel(int32_t* __restrict__ block_hist, int n_chunks, int P,
                                                              int32_t* __restrict__ slot_offsets) {
  __shared__ int wave_sums[kMaxP / 64];
  const int p = threadIdx.x;
  int run = 0;
  if (p < P) {
    // eight independent loads in flight per thread, then the dependent running sum
    int b = 0;
    for (; b + 8 <= n_chunks; b += 8) {
      int v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = block_hist[static_cast<int64_t>(b + j) * P + p];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        block_hist[static_cast<int64_t>(b + j) * P + p] = run;
        run += v[j];
      }
    }
    for (; b < n_chunks; ++b) {
      const int64_t o = static_cast<int64_t>(b) * P + p;
      const int v = block_hist[o];
      block_hist[o] = run;
      run += v;
    }
  }
  // exclusive scan of `run` over the workgroup: wavefront scan, then scan of the wave totals
  const int lane = p & 63, wave = p >> 6;
  int incl = run;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  if (wave == 0) {
    int w = lane < kMaxP / 64 ? wave_sums[lane] : 0;
    int wi = w;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      const int v = __shfl_up(wi, o);
      if (lane >= o) wi += v;
    }
    if (lane < kMaxP / 64) wave_sums[lane] = wi - w;
  }
  __syncthreads();
  const int excl = wave_sums[wave] + incl - run;
  if (p < P) slot_offsets[p] = excl;
  if (p == P - 1) slot_offsets[P] = excl + run;
}

// Stable placement.  Rows of a chunk are visited in ascending index: step s covers rows
// base + s*256 + [0, 256), wavefront w the 64 rows after base + s*256 + w*64.  Inside a wavefront
// the lanes holding the same slot are found with one ballot per bit of the slot id; the lowest
// such lane records the wavefront's count for that slot, counts are prefix-summed over the four
// wavefronts and carried from step to step in `running`.
__global__ __launch_bounds__(kThreads) void dispatch_place_kernel(const int32_t* __restrict__ topk_phys, int N, int P, int nbits,
                                                                  const int32_t* __restrict__ block_base,
                                                                  const int32_t* __restrict__ slot_offsets,
                                                                  int32_t* __restrict__ dst_row, int32_t* __restrict__ src_of) {
  __shared__ int running[kMaxP];
  __shared__ int wave_cnt[kThreads / 64][kMaxP];
  for (int p = threadIdx.x; p < P; p += kThreads) {
    running[p] = slot_offsets[p] + block_base[static_cast<int64_t>(blockIdx.x) * P + p];
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) wave_cnt[w][p] = 0;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int base = blockIdx.x * kChunk;
  for (int s = 0; s < kSteps; ++s) {
    const int i = base + s * kThreads + threadIdx.x;
    int p = -1;
    if (i < N) {
      p = topk_phys[i];
      if (p < 0 || p >= P) p = -1;
    }
    const bool valid = p >= 0;
    unsigned long long peers = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
      const bool bit = (p >> b) & 1;
      const unsigned long long m = __ballot(valid && bit);
      peers &= bit ? m : ~m;
    }
    const unsigned long long below = peers & ((1ull << lane) - 1ull);
    const int rank = __popcll(below);
    const bool leader = valid && below == 0;
    if (leader) wave_cnt[wave][p] = __popcll(peers);
    __syncthreads();
    if (valid) {
      int at = running[p] + rank;
      for (int w = 0; w < wave; ++w) at += wave_cnt[w][p];
      dst_row[i] = at;
      src_of[at] = i;
    } else if (i < N) {
      dst_row[i] = -1;  // slot id outside [0, P): the row is dropped
    }
    __syncthreads();
    if (leader) {
      atomicAdd(&running[p], __popcll(peers));
      wave_cnt[wave][p] = 0;
    }
    __syncthreads();
  }
}

// One workgroup per token; 16-byte words.  The row is read once and written k times.
__global__ __launch_bounds__(kThreads) void dispatch_permute_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ dst_row,
                                                                    int k, int row_words, uint4* __restrict__ x_perm) {
  __shared__ int dst[kMaxK];
  const int t = blockIdx.x;
  if (threadIdx.x < k) dst[threadIdx.x] = dst_row[static_cast<int64_t>(t) * k + threadIdx.x];
  __syncthreads();
  const uint4* src = x + static_cast<int64_t>(t) * row_words;
  for (int c = threadIdx.x; c < row_words; c += kThreads) {
    const uint4 v = src[c];
    for (int j = 0; j < k; ++j) {
      const int d = dst[j];
      if (d >= 0) x_perm[static_cast<int64_t>(d) * row_words + c] = v;
    }
  }
}

}  // namespace

int launch_dispatch(revive_ctx* ctx, const void* x, const int32_t* topk_phys, int T, void* x_perm, int32_t* slot_offsets,
                    int32_t* dst_row, int32_t* src_of, hipStream_t stream) {
  const revive_config& c = ctx->cfg;
  const int P = ctx->P;
  const int N = T * c.k;
  const int n_chunks = ceil_div(N, kChunk);
  int32_t* block_hist = reinterpret_cast<int32_t*>(ctx->d_ws + ctx->ws.off_block_hist);
  int nbits = 1;
  while ((1 << nbits) < P) ++nbits;

  if (n_chunks > 0) {
    KernelTimer timer(ctx, REVIVE_K_DISPATCH_COUNT, stream);
    hipLaunchKernelGGL(dispatch_count_kernel, dim3(n_chunks), dim3(kThreads), 0, stream, topk_phys, N, P, block_hist);
    REVIVE_HIP(ctx, hipGetLastError());
  }
  {
    KernelTimer timer(ctx, REVIVE_K_DISPATCH_SCAN, stream);
    hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(kMaxP), 0, stream, block_hist, n_chunks, P, slot_offsets);
    REVIVE_HIP(ctx, hipGetLastError());
  }
  if (n_chunks > 0) {
    {
      KernelTimer timer(ctx, REVIVE_K_DISPATCH_PLACE, stream);
      hipLaunchKernelGGL(dispatch_place_kernel, dim3(n_chunks), dim3(kThreads), 0, stream, topk_phys, N, P, nbits, block_hist,
                         slot_offsets, dst_row, src_of);
      REVIVE_HIP(ctx, hipGetLastError());
    }
    KernelTimer timer(ctx, REVIVE_K_DISPATCH_PERMUTE, stream);
    const int row_words = static_cast<int>(c.H * ctx->elem / 16);
    hipLaunchKernelGGL(dispatch_permute_kernel, dim3(T), dim3(kThreads), 0, stream, static_cast<const uint4*>(x), dst_row, c.k,
                       row_words, static_cast<uint4*>(x_perm));
    REVIVE_HIP(ctx, hipGetLastError());
  }
  return REVIVE_OK;
}

}  // namespace revive
