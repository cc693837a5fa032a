// Grouped SwiGLU expert FFN of the failure-remapped MoE layer.
//
// Paper: Sec. 2.1 (each expert acts as an FFN).  Every physical slot p that received rows
// [slot_offsets[p], slot_offsets[p+1]) of the permuted activations applies its own weights:
// h = silu(X G_p) * (X U_p), y = h D_p.  Slots without rows (in particular every slot of a failed
// rank, Sec. 3.5) produce no tile, so their weight pointers are never dereferenced.
//
// The row counts exist only on the device, so the launch is shaped by an upper bound: a small
// kernel turns slot_offsets into a list of row-tiles (slot, first row, end row) and the GEMM
// grids cover floor(N / tile) + P tiles; workgroups beyond the list's end exit at once.
#include "gemm_bf16.hpp"
#include "gemm_f32.hpp"

namespace revive {

namespace {

__global__ __launch_bounds__(kMaxP) void ffn_tiles_kernel(const int32_t* __restrict__ slot_offsets, int P, int tile_m,
                                                          const void* const* __restrict__ w_gate_up,
                                                          const void* const* __restrict__ w_down,
                                                          MTile* __restrict__ tiles, int32_t* __restrict__ tile_count) {
  __shared__ int wave_sums[kMaxP / 64];
  __shared__ int tile_base[kMaxP + 1];  // first row-tile of every slot (exclusive prefix sum), [P] = total
  const int p = threadIdx.x;
  int first = 0, end = 0;
  if (p < P) {
    first = slot_offsets[p];
    end = slot_offsets[p + 1];
  }
  const int mine = end > first ? (end - first + tile_m - 1) / tile_m : 0;
  const int lane = p & 63, wave = p >> 6;
  int incl = mine;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  if (wave == 0) {
    const int w = lane < kMaxP / 64 ? wave_sums[lane] : 0;
    int wi = w;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      const int v = __shfl_up(wi, o);
      if (lane >= o) wi += v;
    }
    if (lane < kMaxP / 64) wave_sums[lane] = wi - w;
    if (lane == kMaxP / 64 - 1) tile_count[0] = wi;
  }
  __syncthreads();
  const int base = wave_sums[wave] + incl - mine;
  if (p < P) tile_base[p] = base;
  if (p == P - 1) tile_base[P] = base + mine;
  __syncthreads();
  // One record per row-tile, the records dealt to the threads in order (a slot that holds most of the
  // rows, e.g. when every token picks the same experts, does not leave its thousands of records to one
  // thread).  The slot of record i is the last one whose first record is <= i: a binary search over the
  // prefix sums.  Only slots that received rows have their weight pointers read.
  const int total = tile_base[P];
  for (int i = p; i < total; i += kMaxP) {
    int lo = 0, hi = P - 1;  // invariant: tile_base[lo] <= i, and the answer is in [lo, hi]
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (tile_base[mid] <= i) lo = mid; else hi = mid - 1;
    }
    const int g = lo;  // among slots with equal base (empty ones) the last, which is the one that holds tiles
    MTile t;
    t.group = g;
    t.group_begin = slot_offsets[g];
    t.group_end = slot_offsets[g + 1];
    t.pad = ((tile_base[g + 1] - tile_base[g]) << 16) | (i - tile_base[g]);
    t.w[0] = w_gate_up[g];
    t.w[1] = w_down[g];
    tiles[i] = t;
  }
}

// Tile shapes of the bf16 GEMMs: 256 x 256 outputs per workgroup of 8 wavefronts (2 x 4), K in
// steps of 32 through a four-stage ring of asynchronous global->LDS copies.  Problems too small
// to give every CU a 256 x 256 tile use 256 x 128 tiles on 4 wavefronts (two workgroups per CU).
constexpr int kBM = kTileM_bf16, kBN = 256, kWM = 2, kWN = 4;

struct Bf16Ffn {  // one SwiGLU FFN: rows of A -> h -> y
  const void* A;
  const void* const* gu_tab; const void* gu_one;
  const void* const* dn_tab; const void* dn_one;
  void* h; void* y;
  int I;
  const MTile* tiles; const int32_t* tile_count; int M;
  int max_m_tiles;
  int h_rows;  // rows of the intermediate h, which is kept K-panel-major: [I/32][h_rows][32]
};

GemmArgs gate_up_args(const revive_ctx* ctx, const Bf16Ffn& f, int bn_out) {
  GemmArgs a{};
  a.A = f.A; a.lda = ctx->cfg.H;
  a.B_tab = f.gu_tab; a.B_one = f.gu_one; a.ldb = ctx->cfg.H;
  a.C = f.h; a.ldc = f.I; a.c_rows = f.h_rows;
  a.n_out = f.I; a.K = ctx->cfg.H;
  a.tiles = f.tiles; a.tile_count = f.tile_count; a.M = f.M;
  a.n_col_tiles = ceil_div(f.I, bn_out);
  a.b_sel = f.tiles ? 0 : -1;
  a.b_tiled = 1;
  a.b_rows_pad = ceil_div(f.I, kWeightTileRows) * kWeightTileRows;
  return a;
}

GemmArgs down_args(const revive_ctx* ctx, const Bf16Ffn& f, int bn_out) {
  GemmArgs d{};
  d.A = f.h; d.lda = f.I; d.a_rows = f.h_rows;
  d.B_tab = f.dn_tab; d.B_one = f.dn_one; d.ldb = f.I;
  d.C = f.y; d.ldc = ctx->cfg.H;
  d.n_out = ctx->cfg.H; d.K = f.I;
  d.tiles = f.tiles; d.tile_count = f.tile_count; d.M = f.M;
  d.n_col_tiles = ceil_div(ctx->cfg.H, bn_out);
  d.b_sel = f.tiles ? 1 : -1;
  d.b_tiled = 1;
  d.b_rows_pad = ceil_div(ctx->cfg.H, kWeightTileRows) * kWeightTileRows;
  return d;
}

// Runs one FFN, or two in the same pair of launches (their tiles share the grid, which shortens
// the partially filled last round of workgroups).  K_GATE_UP / K_DOWN name the launches.
template <int K_GATE_UP, int K_DOWN>
int bf16_ffn(revive_ctx* ctx, const Bf16Ffn& f0, const Bf16Ffn* f1, hipStream_t stream) {
  const int H = ctx->cfg.H;
  const int64_t tiles_big_down = static_cast<int64_t>(f0.max_m_tiles) * ceil_div(H, kBN) +
                                 (f1 ? static_cast<int64_t>(f1->max_m_tiles) * ceil_div(H, kBN) : 0);
  const bool small = !f1 && f0.tiles == nullptr && tiles_big_down < 2 * 256;  // dense and under two tiles per CU
  {
    KernelTimer timer(ctx, K_GATE_UP, stream);
    int rc;
    if (small) {
      GemmArgs a0 = gate_up_args(ctx, f0, 64);
      rc = launch_gemm_bf16_dma<kBM, 128, 2, 2, EPI_SWIGLU, K_GATE_UP>(ctx, a0, f0.max_m_tiles, nullptr, 0, stream);
    } else {
      GemmArgs a0 = gate_up_args(ctx, f0, kBN / 2), a1{};
      if (f1) a1 = gate_up_args(ctx, *f1, kBN / 2);
      rc = launch_gemm_bf16_dma<kBM, kBN, kWM, kWN, EPI_SWIGLU, K_GATE_UP>(ctx, a0, f0.max_m_tiles, f1 ? &a1 : nullptr,
                                                                           f1 ? f1->max_m_tiles : 0, stream);
    }
    if (rc != REVIVE_OK) return rc;
  }
  KernelTimer timer(ctx, K_DOWN, stream);
  if (small) {
    GemmArgs d0 = down_args(ctx, f0, 128);
    return launch_gemm_bf16_dma<kBM, 128, 2, 2, EPI_BF16, K_DOWN>(ctx, d0, f0.max_m_tiles, nullptr, 0, stream);
  }
  GemmArgs d0 = down_args(ctx, f0, kBN), d1{};
  if (f1) d1 = down_args(ctx, *f1, kBN);
  return launch_gemm_bf16_dma<kBM, kBN, kWM, kWN, EPI_BF16, K_DOWN>(ctx, d0, f0.max_m_tiles, f1 ? &d1 : nullptr,
                                                                    f1 ? f1->max_m_tiles : 0, stream);
}

template <int K_GATE_UP, int K_DOWN>
int f32_gemm_pair(revive_ctx* ctx, const void* A, const void* const* gu_tab, const void* gu_one, const void* const* dn_tab,
                  const void* dn_one, void* h, void* y, int I, const MTile* tiles, const int32_t* tile_count, int M,
                  int max_m_tiles, hipStream_t stream) {
  const int H = ctx->cfg.H;
  GemmF32Args a{};
  a.A = static_cast<const float*>(A); a.lda = H;
  a.B_tab = gu_tab; a.B_one = static_cast<const float*>(gu_one); a.ldb = H;
  a.C = static_cast<float*>(h); a.ldc = I;
  a.n_out = I; a.K = H;
  a.tiles = tiles; a.tile_count = tile_count; a.M = M;
  a.n_col_tiles = ceil_div(I, 64);
  {
    KernelTimer timer(ctx, K_GATE_UP, stream);
    int rc = launch_gemm_f32<true>(ctx, a, max_m_tiles, stream);
    if (rc != REVIVE_OK) return rc;
  }
  GemmF32Args d{};
  d.A = static_cast<const float*>(h); d.lda = I;
  d.B_tab = dn_tab; d.B_one = static_cast<const float*>(dn_one); d.ldb = I;
  d.C = static_cast<float*>(y); d.ldc = H;
  d.n_out = H; d.K = I;
  d.tiles = tiles; d.tile_count = tile_count; d.M = M;
  d.n_col_tiles = ceil_div(H, 64);
  KernelTimer timer(ctx, K_DOWN, stream);
  return launch_gemm_f32<false>(ctx, d, max_m_tiles, stream);
}

}  // namespace

int launch_expert_ffn(revive_ctx* ctx, const void* x_perm, const int32_t* slot_offsets, const void* const* w_gate_up,
                      const void* const* w_down, void* y_perm, const void* x, const void* w_sh_gate_up, const void* w_sh_down,
                      void* y_shared, int T, hipStream_t stream) {
  const revive_config& c = ctx->cfg;
  const bool bf16 = c.dtype == REVIVE_DTYPE_BF16;
  const int tile_m = bf16 ? kTileM_bf16 : kTileM_f32;
  const int64_t N = static_cast<int64_t>(T) * c.k;
  MTile* tiles = reinterpret_cast<MTile*>(ctx->d_ws + ctx->ws.off_tiles);
  int32_t* tile_count = reinterpret_cast<int32_t*>(ctx->d_ws + ctx->ws.off_tile_count);
  void* h = ctx->d_ws + ctx->ws.off_h;
  {
    KernelTimer timer(ctx, REVIVE_K_FFN_TILES, stream);
    hipLaunchKernelGGL(ffn_tiles_kernel, dim3(1), dim3(kMaxP), 0, stream, slot_offsets, ctx->P, tile_m, w_gate_up, w_down, tiles,
                       tile_count);
    REVIVE_HIP(ctx, hipGetLastError());
  }
  const int bound = max_tiles(N, ctx->P, tile_m);
  constexpr int GU = REVIVE_K_FFN_GATE_UP, DN = REVIVE_K_FFN_DOWN;
  if (bf16) {
    Bf16Ffn routed{x_perm, w_gate_up, nullptr, w_down, nullptr, h, y_perm, c.I, tiles, tile_count, 0, bound, static_cast<int>(N)};
    if (!y_shared) return bf16_ffn<GU, DN>(ctx, routed, nullptr, stream);
    // routed and shared experts in the same two launches
    Bf16Ffn shared{x, nullptr, w_sh_gate_up, nullptr, w_sh_down, ctx->d_ws + ctx->ws.off_h_shared, y_shared, c.I_shared,
                   nullptr, nullptr, T, ceil_div(T, tile_m), T};
    return bf16_ffn<GU, DN>(ctx, routed, &shared, stream);
  }
  int rc = f32_gemm_pair<GU, DN>(ctx, x_perm, w_gate_up, nullptr, w_down, nullptr, h, y_perm, c.I, tiles, tile_count, 0, bound, stream);
  if (rc != REVIVE_OK || !y_shared) return rc;
  return launch_shared_ffn(ctx, x, w_sh_gate_up, w_sh_down, y_shared, T, stream);
}

int launch_shared_ffn(revive_ctx* ctx, const void* x, const void* w_sh_gate_up, const void* w_sh_down, void* y_shared, int T,
                      hipStream_t stream) {
  const revive_config& c = ctx->cfg;
  const bool bf16 = c.dtype == REVIVE_DTYPE_BF16;
  const int dense_tiles = ceil_div(T, bf16 ? kTileM_bf16 : kTileM_f32);
  void* h_shared = ctx->d_ws + ctx->ws.off_h_shared;
  constexpr int SGU = REVIVE_K_FFN_SHARED_GATE_UP, SDN = REVIVE_K_FFN_SHARED_DOWN;
  if (bf16) {
    Bf16Ffn shared{x, nullptr, w_sh_gate_up, nullptr, w_sh_down, h_shared, y_shared, c.I_shared, nullptr, nullptr, T, dense_tiles, T};
    return bf16_ffn<SGU, SDN>(ctx, shared, nullptr, stream);
  }
  return f32_gemm_pair<SGU, SDN>(ctx, x, nullptr, w_sh_gate_up, nullptr, w_sh_down, h_shared, y_shared, c.I_shared, nullptr, nullptr, T, dense_tiles, stream);
}

}  // namespace revive
