// Grouped fp32 GEMM (vector FMA, fp32 accumulate) for the fp32 layer configuration.
//
// Same contract as the bf16 kernel: C[row, n] = sum_k A[row, k] * B_group[n, k], with row-tiles
// that each belong to one group, and an optional fused SwiGLU (B holds gate rows then up rows).
// 64x64 output tile per 256-thread workgroup, 4x4 outputs per thread, K walked in steps of 16
// through LDS.  This path exists for correctness at small fp32 shapes, not for speed.
#pragma once

#include <hip/hip_runtime.h>

#include "ctx.hpp"

namespace revive {

struct GemmF32Args {
  const float* A;
  int64_t lda;
  const void* const* B_tab;
  const float* B_one;
  int64_t ldb;
  float* C;
  int64_t ldc;
  int n_out;
  int K;  // multiple of 4
  const MTile* tiles;
  const int32_t* tile_count;
  int M;
  int n_col_tiles;
};

template <bool SWIGLU>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmF32Args g) {
  constexpr int BM = kTileM_f32, BN = 64, BK = 16, LD = 68;
  __shared__ float As[BK][LD];
  __shared__ float Bs[SWIGLU ? 2 : 1][BK][LD];

  const int n_m_tiles = g.tiles ? *g.tile_count : (g.M + BM - 1) / BM;
  const int m_idx = blockIdx.x / g.n_col_tiles;
  const int n_idx = blockIdx.x - m_idx * g.n_col_tiles;
  if (m_idx >= n_m_tiles) return;
  int group = 0, row_begin, row_end;
  if (g.tiles) {
    const MTile t = g.tiles[m_idx];
    group = t.group;
    tile_span(t.group_begin, t.group_end, t.pad >> 16, t.pad & 0xFFFF, BM, row_begin, row_end);
  } else {
    row_begin = m_idx * BM;
    row_end = min(g.M, row_begin + BM);
  }
  const float* B = g.B_tab ? static_cast<const float*>(g.B_tab[group]) : g.B_one;
  const int n0 = n_idx * BN;

  const int tid = threadIdx.x;
  const int lrow = tid >> 2, lk = (tid & 3) * 4;  // this thread's row and k-quad of the tile loads
  const int arow = min(row_begin + lrow, row_end - 1);
  const int bcol = min(n0 + lrow, g.n_out - 1);
  const float* a_src = g.A + static_cast<int64_t>(arow) * g.lda + lk;
  const float* b_src = B + static_cast<int64_t>(bcol) * g.ldb + lk;
  const float* u_src = B + static_cast<int64_t>(bcol + g.n_out) * g.ldb + lk;

  const int tx = tid & 15, ty = tid >> 4;  // 4 columns tx*4.., 4 rows ty*4..
  float acc[4][4] = {}, accu[4][4] = {};

  for (int k0 = 0; k0 < g.K; k0 += BK) {
    const bool in = k0 + lk < g.K;
    float4 av = in ? *reinterpret_cast<const float4*>(a_src + k0) : make_float4(0, 0, 0, 0);
    float4 bv = in ? *reinterpret_cast<const float4*>(b_src + k0) : make_float4(0, 0, 0, 0);
    As[lk + 0][lrow] = av.x; As[lk + 1][lrow] = av.y; As[lk + 2][lrow] = av.z; As[lk + 3][lrow] = av.w;
    Bs[0][lk + 0][lrow] = bv.x; Bs[0][lk + 1][lrow] = bv.y; Bs[0][lk + 2][lrow] = bv.z; Bs[0][lk + 3][lrow] = bv.w;
    if (SWIGLU) {
      float4 uv = in ? *reinterpret_cast<const float4*>(u_src + k0) : make_float4(0, 0, 0, 0);
      Bs[1][lk + 0][lrow] = uv.x; Bs[1][lk + 1][lrow] = uv.y; Bs[1][lk + 2][lrow] = uv.z; Bs[1][lk + 3][lrow] = uv.w;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4], u[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[0][kk][tx * 4 + j];
      if (SWIGLU) {
#pragma unroll
        for (int j = 0; j < 4; ++j) u[j] = Bs[1][kk][tx * 4 + j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
          if (SWIGLU) accu[i][j] = fmaf(a[i], u[j], accu[i][j]);
        }
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = row_begin + ty * 4 + i;
    if (row >= row_end) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      if (col >= g.n_out) continue;
      float v = acc[i][j];
      if (SWIGLU) v = v / (1.0f + expf(-v)) * accu[i][j];
      g.C[static_cast<int64_t>(row) * g.ldc + col] = v;
    }
  }
}

template <bool SWIGLU>
int launch_gemm_f32(revive_ctx* ctx, const GemmF32Args& args, int max_m_tiles, hipStream_t stream) {
  const int64_t total = static_cast<int64_t>(max_m_tiles) * args.n_col_tiles;
  if (total <= 0) return REVIVE_OK;
  hipLaunchKernelGGL(gemm_f32_kernel<SWIGLU>, dim3(static_cast<unsigned>(total)), dim3(256), 0, stream, args);
  return check_hip(ctx, hipGetLastError(), "gemm_f32 launch");
}

}  // namespace revive
