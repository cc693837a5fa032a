// Dispatch (A2E) of the failure-remapped MoE layer: a deterministic stable counting sort of the
// routed rows by physical slot, then the row permutation.
//
// Paper: Sec. 2.3 (dispatch routes tokens to their top-k experts).  Slots are laid out rank by
// rank, so the sorted buffer is rank-segmented: segment r is what rank r would receive.  A failed
// rank's slots never appear in topk_phys (Sec. 3.4), so its segment is empty (Sec. 3.5).
//
// Two kernels, both with grids fixed by T:
//   index    per chunk of 1024 routed rows: stable rank of every row among the rows of its slot
//            in the chunk (-> dst_row, for now) and the chunk's histogram -> block_hist[chunk][P];
//            the workgroup that finishes last turns the columns into running sums over the
//            chunks and scans the totals over P -> block_hist (bases), slot_offsets
//   permute  one workgroup per token: destination of each of its k routed rows = slot offset +
//            chunk base + rank in the chunk (-> dst_row, src_of), then the row is read once and
//            written to its k destinations
#include <mutex>

#include "ctx.hpp"

namespace revive {

namespace {

constexpr int kChunk = kDispatchChunk;  // routed rows per workgroup of the index kernel
constexpr int kThreads = 256;

// One workgroup of kMaxP threads per chunk: a thread handles one routed row of the histogram and,
// in the workgroup that finishes last, one slot column of the scan.
// `ticket` counts finished workgroups; the last one resets it, so it is zero between launches.
__global__ __launch_bounds__(kMaxP) void dispatch_index_kernel(const int32_t* __restrict__ topk_phys, int N, int P, int nbits,
                                                               int32_t* block_hist, int32_t* __restrict__ slot_offsets,
                                                               int32_t* __restrict__ rank_in_chunk, unsigned int* ticket) {
  static_assert(kChunk == kMaxP, "one routed row and one slot column per thread");
  constexpr int kWaves = kMaxP / 64;
  __shared__ uint8_t wave_cnt[kWaves][kMaxP];  // rows of a slot held by each 64-row wavefront of the chunk (<= 64)
  __shared__ int wave_sums[kWaves];
  __shared__ int last_flag;
  const int p = threadIdx.x;
  const int lane = p & 63, wave = p >> 6;
  for (int j = p; j < kWaves * P; j += kMaxP) wave_cnt[j / P][j % P] = 0;
  __syncthreads();
  // Rows are taken in ascending index: wavefront w holds rows [64w, 64w + 64) of the chunk.  The
  // lanes that hold the same slot are found with one ballot per bit of the slot id.
  const int i = blockIdx.x * kChunk + threadIdx.x;
  int q = -1;
  if (i < N) {
    q = topk_phys[i];
    if (q < 0 || q >= P) q = -1;  // slot id outside [0, P): the row is dropped
  }
  const bool valid = q >= 0;
  unsigned long long peers = __ballot(valid);
  for (int b = 0; b < nbits; ++b) {
    const bool bit = (q >> b) & 1;
    const unsigned long long m = __ballot(valid && bit);
    peers &= bit ? m : ~m;
  }
  const unsigned long long below = peers & ((1ull << lane) - 1ull);
  if (valid && below == 0) wave_cnt[wave][q] = static_cast<uint8_t>(__popcll(peers));
  __syncthreads();
  if (i < N) {
    int r = -1;
    if (valid) {
      r = __popcll(below);
      for (int w = 0; w < wave; ++w) r += wave_cnt[w][q];
    }
    rank_in_chunk[i] = r;
  }
  if (p < P) {
    int total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) total += wave_cnt[w][p];
    block_hist[static_cast<int64_t>(blockIdx.x) * P + p] = total;
  }

  // Publish this chunk's histogram and ranks device-wide, then take a ticket; only the workgroup
  // holding the last ticket goes on (nobody waits for anybody).
  //
  // What makes the other workgroups' stores visible to the last one.  The release and the acquire
  // of an agent-scope atomic are cache operations, not per-wavefront ones: the release writes the
  // dirty lines of this XCD's L2 back to the memory the XCDs share, whichever wavefront stored
  // them, and the acquire invalidates the compute unit's L1 (and what this XCD's L2 holds of
  // lines another XCD may have written), for every wavefront that loads afterwards.  So one
  // thread issues them for the workgroup, provided that (1) every wavefront's own stores have
  // reached L2 before the release: the vmcnt wait below (stores count in vmcnt on gfx9), then the
  // barrier; and (2) no wavefront loads before the acquire: the second barrier.  This is stronger
  // than what the HIP memory model promises for a fence issued by one thread; the portable form,
  // an agent-scope release and acquire fence in every wavefront, was measured and costs one more
  // L2 write-back per wavefront: 12.7 instead of 4.5 us at 24 chunks.
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
  int incl = run;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int u = __shfl_up(incl, o);
    if (lane >= o) incl += u;
  }
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  if (wave == 0) {
    const int w = lane < kWaves ? wave_sums[lane] : 0;
    int wi = w;
#pragma unroll
    for (int o = 1; o < kWaves; o <<= 1) {
      const int u = __shfl_up(wi, o);
      if (lane >= o) wi += u;
    }
    if (lane < kWaves) wave_sums[lane] = wi - w;
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
//   slot_offsets[p] + (rows of slot p in earlier chunks) + (rank of i among the rows of slot p in its chunk),
// the position a stable counting sort by slot gives it.  dst_row arrives holding the rank (or -1).
__global__ __launch_bounds__(kThreads) void dispatch_permute_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ topk_phys,
                                                                    int k, int P, const int32_t* __restrict__ block_base,
                                                                    const int32_t* __restrict__ slot_offsets, int row_words,
                                                                    int32_t* __restrict__ dst_row, int32_t* __restrict__ src_of,
                                                                    uint4* __restrict__ x_perm) {
  __shared__ int dst[kMaxK];
  const int t = blockIdx.x;
  if (threadIdx.x < k) {
    const int i = t * k + threadIdx.x;
    const int r = dst_row[i];
    int d = -1;
    if (r >= 0) {
      const int p = topk_phys[i];
      d = slot_offsets[p] + block_base[static_cast<int64_t>(i / kChunk) * P + p] + r;
      src_of[d] = i;
      dst_row[i] = d;
    }
    dst[threadIdx.x] = d;
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

// Compacted rank segments (Sec. 3.5): after the failed ranks have left the communication domain the
// survivors are renumbered 0 .. n_live-1 in their old order; segment l of the permuted buffer is the
// rows of the rank that now holds logical rank l.  Failed ranks received no rows, so the compacted
// segments tile [0, N) without gaps; entries n_live .. R all hold N.
__global__ __launch_bounds__(256) void rank_offsets_kernel(const int32_t* __restrict__ slot_offsets,
                                                           const int32_t* __restrict__ logical_rank,
                                                           const int32_t* __restrict__ n_live_ranks, int R, int S,
                                                           int32_t* __restrict__ rank_offsets) {
  const int n_live = n_live_ranks[0];
  const int total = slot_offsets[R * S];
  for (int r = threadIdx.x; r <= R; r += 256) {
    if (r < R) {
      const int l = logical_rank[r];
      if (l >= 0) rank_offsets[l] = slot_offsets[r * S];
    }
    if (r >= n_live) rank_offsets[r] = total;
  }
}

}  // namespace

int launch_rank_offsets(revive_ctx* ctx, const int32_t* slot_offsets, int32_t* rank_offsets, hipStream_t stream) {
  hipLaunchKernelGGL(rank_offsets_kernel, dim3(1), dim3(256), 0, stream, slot_offsets, ctx->d_logical_rank(), ctx->d_n_live_ranks(),
                     ctx->cfg.n_ranks, ctx->cfg.slots_per_rank, rank_offsets);
  return check_hip(ctx, hipGetLastError(), "rank_offsets launch");
}

// The two dispatch kernels with their scratch (chunk histograms, ticket) at the given addresses.
static int run_dispatch(revive_ctx* ctx, const void* x, const int32_t* topk_phys, int T, void* x_perm, int32_t* slot_offsets,
                        int32_t* dst_row, int32_t* src_of, int32_t* block_hist, unsigned int* ticket, hipStream_t stream) {
  const revive_config& c = ctx->cfg;
  const int P = ctx->P;
  const int N = T * c.k;
  const int n_chunks = ceil_div(N, kChunk);
  int nbits = 1;
  while ((1 << nbits) < P) ++nbits;
  {
    // with no rows one workgroup still runs, so that slot_offsets becomes all zero
    KernelTimer timer(ctx, REVIVE_K_DISPATCH_INDEX, stream);
    hipLaunchKernelGGL(dispatch_index_kernel, dim3(n_chunks > 0 ? n_chunks : 1), dim3(kMaxP), 0, stream, topk_phys, N, P, nbits,
                       block_hist, slot_offsets, dst_row, ticket);
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

int launch_dispatch(revive_ctx* ctx, const void* x, const int32_t* topk_phys, int T, void* x_perm, int32_t* slot_offsets,
                    int32_t* dst_row, int32_t* src_of, hipStream_t stream) {
  return run_dispatch(ctx, x, topk_phys, T, x_perm, slot_offsets, dst_row, src_of,
                      reinterpret_cast<int32_t*>(ctx->d_ws + ctx->ws.off_block_hist),
                      reinterpret_cast<unsigned int*>(ctx->d_ws + ctx->ws.off_ticket), stream);
}

// ---- dispatch without any allocation: the scratch is a static device array ---------------------
//
// For callers that cannot allocate or bind a workspace.  The array lives in every GPU the library
// is loaded on until the process ends; each device has its own copy at its own address, which is
// looked up once per device (the array's name itself is not a device address in host code).

namespace {

constexpr size_t kStaticHistBytes = sizeof(int32_t) * static_cast<size_t>(kStaticDispatchChunks) * kMaxP;
constexpr size_t kStaticTicketOffset = kStaticHistBytes;  // a multiple of 256
constexpr size_t kStaticScratchBytes = kStaticHistBytes + 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char* g_scratch_ptr[kMaxDevices] = {nullptr};

__global__ void clear_word_kernel(unsigned int* word) { *word = 0u; }

}  // namespace

int init_static_dispatch_scratch(revive_ctx* ctx) {
  int dev = 0;
  REVIVE_HIP(ctx, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(ctx, REVIVE_EINVAL, "device %d: more devices than the library keeps scratch pointers for", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev]) return REVIVE_OK;
  void* p = nullptr;
  REVIVE_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
  if (!p) return fail(ctx, REVIVE_EHIP, "hipGetSymbolAddress returned a null address for the dispatch scratch");
  g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  return REVIVE_OK;
}

int launch_dispatch_static(revive_ctx* ctx, const void* x, const int32_t* topk_phys, int T, void* x_perm, int32_t* slot_offsets,
                           int32_t* dst_row, int32_t* src_of, hipStream_t stream) {
  const int64_t N = static_cast<int64_t>(T) * ctx->cfg.k;
  if (N > static_cast<int64_t>(kStaticDispatchChunks) * kChunk)
    return fail(ctx, REVIVE_EINVAL, "revive_dispatch_static: T * k = %lld routed rows, the static scratch holds at most %d",
                static_cast<long long>(N), kStaticDispatchChunks * kChunk);
  int dev = 0;
  REVIVE_HIP(ctx, hipGetDevice(&dev));
  unsigned char* base = nullptr;  // this device's copy of the array (never the array's name: that is a host-side stand-in)
  if (dev >= 0 && dev < kMaxDevices) {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    base = g_scratch_ptr[dev];
  }
  if (!base) return fail(ctx, REVIVE_ESTATE, "revive_dispatch_static: no context has been created on device %d", dev);
  unsigned int* ticket = reinterpret_cast<unsigned int*>(base + kStaticTicketOffset);
  // the array keeps whatever the previous call left: the ticket must start at zero (a fill kernel,
  // not a memset node, so that the call can be recorded into a graph); the histograms are
  // overwritten before they are read
  hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, stream, ticket);
  REVIVE_HIP(ctx, hipGetLastError());
  return run_dispatch(ctx, x, topk_phys, T, x_perm, slot_offsets, dst_row, src_of, reinterpret_cast<int32_t*>(base), ticket, stream);
}

}  // namespace revive
