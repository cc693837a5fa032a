// Dispatch (A2E) of the failure-remapped MoE layer: a deterministic stable counting sort of the
// routed rows by physical slot, then the row permutation.
//
// Paper: Sec. 2.3 (dispatch routes tokens to their top-k experts).  Slots are laid out rank by
// rank, so the sorted buffer is rank-segmented: segment r is what rank r would receive.  A failed
// rank's slots never appear in topk_phys (Sec. 3.4), so its segment is empty (Sec. 3.5).
//
// Two kernels, both with grids fixed by T:
//   index    per-chunk LDS histogram of the slot ids -> block_hist[chunk][P]; the workgroup that
//            finishes last turns the columns into running sums over the chunks and scans the
//            totals over P -> block_hist (bases), slot_offsets
//   permute  one workgroup per token: stable destination of each of its k routed rows (rows of
//            the same chunk and slot that come before it are counted from topk_phys, which is
//            L2-resident), then the row is read once and written to its k destinations
#include "ctx.hpp"

namespace revive {

namespace {

constexpr int kChunk = kDispatchChunk;  // routed rows per workgroup of the index kernel
constexpr int kThreads = 256;
static_assert(kMaxK < kChunk, "a token's rows touch at most two chunks");

// One workgroup of kMaxP threads per chunk: a thread handles one routed row of the histogram and,
// in the workgroup that finishes last, one slot column of the scan.
// `ticket` counts finished workgroups; the last one resets it, so it is zero between launches.
__global__ __launch_bounds__(kMaxP) void dispatch_index_kernel(const int32_t* __restrict__ topk_phys, int N, int P,
                                                               int32_t* block_hist, int32_t* __restrict__ slot_offsets,
                                                               unsigned int* ticket) {
  static_assert(kChunk == kMaxP, "one routed row and one slot column per thread");
  __shared__ int hist[kMaxP];
  __shared__ int wave_sums[kMaxP / 64];
  __shared__ int last_flag;
  const int p = threadIdx.x;
  hist[p] = 0;
  __syncthreads();
  const int i = blockIdx.x * kChunk + threadIdx.x;
  if (i < N) {
    const int q = topk_phys[i];
    if (q >= 0 && q < P) atomicAdd(&hist[q], 1);
  }
  __syncthreads();
  if (p < P) block_hist[static_cast<int64_t>(blockIdx.x) * P + p] = hist[p];

  // Publish this chunk's histogram device-wide, then take a ticket; only the workgroup holding the
  // last ticket goes on (nobody waits for anybody).  The barrier orders the workgroup's stores
  // before thread 0's release, and thread 0's acquire before the workgroup's later loads; one
  // thread does the device-scope part because each such fence is a cache operation of its own.
  // Every wavefront first waits until its own stores have been accepted by L2.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0)
    last_flag = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1;
  __syncthreads();
  if (!last_flag) return;

  // Column p of block_hist becomes exclusive running sums over the chunks (the rows of slot p that
  // earlier chunks hold); `run` ends as the column total.
  const int n_chunks = gridDim.x;
  int run = 0;
  if (p < P) {
    int b = 0;
    for (; b + 8 <= n_chunks; b += 8) {  // eight independent loads in flight, then the dependent sums
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
  // exclusive scan of `run` over the slots: wavefront scan, then scan of the wavefront totals
  const int lane = p & 63, wave = p >> 6;
  int incl = run;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int u = __shfl_up(incl, o);
    if (lane >= o) incl += u;
  }
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  if (wave == 0) {
    const int w = lane < kMaxP / 64 ? wave_sums[lane] : 0;
    int wi = w;
#pragma unroll
    for (int o = 1; o < kMaxP / 64; o <<= 1) {
      const int u = __shfl_up(wi, o);
      if (lane >= o) wi += u;
    }
    if (lane < kMaxP / 64) wave_sums[lane] = wi - w;
  }
  __syncthreads();
  const int excl = wave_sums[wave] + incl - run;
  if (p < P) slot_offsets[p] = excl;
  if (p == P - 1) {
    slot_offsets[P] = excl + run;  // number of valid routed rows
    *ticket = 0;
  }
}

// One workgroup per token; 16-byte words.  Routed row i = t*k + j goes to
//   slot_offsets[p] + (rows of slot p in earlier chunks) + (rows of slot p earlier in i's chunk),
// the position a stable counting sort by slot gives it.
__global__ __launch_bounds__(kThreads) void dispatch_permute_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ topk_phys,
                                                                    int k, int P, const int32_t* __restrict__ block_base,
                                                                    const int32_t* __restrict__ slot_offsets, int row_words,
                                                                    int32_t* __restrict__ dst_row, int32_t* __restrict__ src_of,
                                                                    uint4* __restrict__ x_perm) {
  __shared__ int slot[kMaxK], cnt[kMaxK], dst[kMaxK];
  const int t = blockIdx.x;
  const int i0 = t * k;
  if (threadIdx.x < k) {
    int p = topk_phys[i0 + threadIdx.x];
    if (p < 0 || p >= P) p = -1;  // slot id outside [0, P): the row is dropped
    slot[threadIdx.x] = p;
    cnt[threadIdx.x] = 0;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int first = (i0 / kChunk) * kChunk;  // start of the chunk that holds row i0
  const int last_row = i0 + k - 1;
  for (int b = first; b < last_row; b += kThreads) {
    const int idx = b + threadIdx.x;
    const int v = idx < last_row ? topk_phys[idx] : -1;
    for (int j = 0; j < k; ++j) {
      const int ij = i0 + j;
      const int start_j = (ij / kChunk) * kChunk;
      const bool hit = v >= 0 && v == slot[j] && idx >= start_j && idx < ij;
      const unsigned long long m = __ballot(hit);
      if (lane == 0 && m) atomicAdd(&cnt[j], __popcll(m));
    }
  }
  __syncthreads();
  if (threadIdx.x < k) {
    const int p = slot[threadIdx.x];
    const int i = i0 + threadIdx.x;
    int d = -1;
    if (p >= 0) {
      d = slot_offsets[p] + block_base[static_cast<int64_t>(i / kChunk) * P + p] + cnt[threadIdx.x];
      src_of[d] = i;
    }
    dst[threadIdx.x] = d;
    dst_row[i] = d;
  }
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
  unsigned int* ticket = reinterpret_cast<unsigned int*>(ctx->d_ws + ctx->ws.off_ticket);
  {
    // with no rows one workgroup still runs, so that slot_offsets becomes all zero
    KernelTimer timer(ctx, REVIVE_K_DISPATCH_INDEX, stream);
    hipLaunchKernelGGL(dispatch_index_kernel, dim3(n_chunks > 0 ? n_chunks : 1), dim3(kMaxP), 0, stream, topk_phys, N, P,
                       block_hist, slot_offsets, ticket);
    REVIVE_HIP(ctx, hipGetLastError());
  }
  if (T > 0) {
    KernelTimer timer(ctx, REVIVE_K_DISPATCH_PERMUTE, stream);
    const int row_words = static_cast<int>(c.H * ctx->elem / 16);
    hipLaunchKernelGGL(dispatch_permute_kernel, dim3(T), dim3(kThreads), 0, stream, static_cast<const uint4*>(x), topk_phys, c.k, P,
                       block_hist, slot_offsets, row_words, dst_row, src_of, static_cast<uint4*>(x_perm));
    REVIVE_HIP(ctx, hipGetLastError());
  }
  return REVIVE_OK;
}

}  // namespace revive
